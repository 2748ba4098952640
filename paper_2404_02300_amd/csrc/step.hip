// sdt_train_step: one mini-batch of GraphSAGE-mean training on the worker's
// partition, enqueued on one stream with no host synchronisation.  All
// data-dependent sizes (frontier sizes, edge counts) stay in device memory;
// every kernel is launched for the upper bound and reads the true count.
#include <vector>
#include <mutex>
#include "common.h"

#include <atomic>
#include <string>
#include <thread>

namespace sdt {
namespace {

struct Caps {
    int32_t dst[SDT_MAX_LAYERS], src[SDT_MAX_LAYERS], nnz[SDT_MAX_LAYERS];
};

bool compute_caps(int64_t n_nodes, int32_t batch, const int32_t* fanouts, int L, Caps* c) {
    int64_t dst = batch;
    for (int l = L - 1; l >= 0; --l) {
        const int64_t nnz = dst * fanouts[l];
        int64_t src = dst + nnz;
        if (src > n_nodes) src = n_nodes;
        if (src < dst) src = dst;
        if (nnz > 0x7FFFFFFF || src > 0x7FFFFFFF) return false;
        c->dst[l] = (int32_t)dst;
        c->nnz[l] = (int32_t)nnz;
        c->src[l] = (int32_t)src;
        dst = src;
    }
    return true;
}

// width of one of the two operands the projection kernels take: [Hself | A] for GraphSAGE, the two
// halves of the aggregated row for GCN (whose single weight matrix [in, out] is then [2 * in/2, out])
inline int32_t operand_width(const sdt_model* m, int l) { return m->kind != SDT_MODEL_SAGE_MEAN ? m->dims[l] / 2 : m->dims[l]; }

// scratch of one layer's projection backward (split partials of dW/db, or the fused head's)
size_t bwd_scratch_bytes(int32_t batch, int32_t cap_dst, int32_t in, int32_t out, bool last) {
    // (sized for the split-bf16 weight gradient where the shape suits it: at least the plain path's need)
    size_t lb = linear_bwd_workspace_bytes_x3(cap_dst, in, out);
    const size_t plain = sdt_linear_bwd_workspace_bytes(cap_dst, in, out);
    if (plain > lb) lb = plain;
    // the forward of the same layer may borrow the region first (partial tiles of the split-bf16 projection)
    const size_t fb = last ? 0 : x3_fwd_workspace_bytes(cap_dst, in, out);
    if (fb > lb) lb = fb;
    if (last && head_supported(in, out)) {
        const size_t hb = head_workspace_bytes(batch, in, out);
        if (hb > lb) lb = hb;
    }
    return align_up(lb, 256);
}

int32_t check_model(const sdt_model* m, const int32_t* fanouts, const char* who) {
    SDT_REQUIRE(m && fanouts, SDT_ERR_INVALID_ARG, "%s: null model or fanouts", who);
    SDT_REQUIRE(m->n_layers >= 1 && m->n_layers <= SDT_MAX_LAYERS, SDT_ERR_INVALID_ARG, "%s: n_layers %d outside [1,%d]",
                who, m->n_layers, SDT_MAX_LAYERS);
    for (int l = 0; l <= m->n_layers; ++l)
        SDT_REQUIRE(m->dims[l] > 0, SDT_ERR_INVALID_ARG, "%s: dims[%d] = %d", who, l, m->dims[l]);
    for (int l = 0; l < m->n_layers; ++l)
        SDT_REQUIRE(fanouts[l] >= 0 && fanouts[l] <= SDT_MAX_FANOUT, SDT_ERR_INVALID_ARG,
                    "%s: fanouts[%d] = %d outside [0,%d]", who, l, fanouts[l], SDT_MAX_FANOUT);
    SDT_REQUIRE(m->kind == SDT_MODEL_SAGE_MEAN || m->kind == SDT_MODEL_GCN || m->kind == SDT_MODEL_GAT, SDT_ERR_INVALID_ARG,
                "%s: unknown model kind %d", who, m->kind);
    if (m->kind != SDT_MODEL_SAGE_MEAN)
        for (int l = 0; l < m->n_layers; ++l)
            SDT_REQUIRE(m->dims[l] % 2 == 0, SDT_ERR_INVALID_ARG,
                        "%s: GCN and GAT need even layer input widths (dims[%d] = %d): the projection runs as two half-width operands",
                        who, l, m->dims[l]);
    if (m->kind == SDT_MODEL_GAT)
        SDT_REQUIRE(m->gat_slope >= 0.f && m->gat_slope <= 1.f, SDT_ERR_INVALID_ARG, "%s: gat_slope %g outside [0,1]", who,
                    (double)m->gat_slope);
    return SDT_OK;
}

}  // namespace
}  // namespace sdt

using namespace sdt;

extern "C" size_t sdt_struct_bytes(int32_t which) {
    switch (which) {
        case 0: return sizeof(sdt_csr);
        case 1: return sizeof(sdt_block);
        case 2: return sizeof(sdt_model);
        case 3: return sizeof(sdt_step_layout);
        case 4: return sizeof(sdt_partition);
        default: return 0;
    }
}

// ---- per-stage HIP-event timing (the object and its recorder are in common.h) -----
static int32_t timing_create(int32_t max_steps, const uint64_t* mask, sdt_timing** out) {
    SDT_REQUIRE(out && mask && max_steps > 0 && max_steps <= (1 << 20), SDT_ERR_INVALID_ARG, "sdt_timing_create: bad arguments");
    sdt_timing* t = new sdt_timing();
    t->max_steps = max_steps;
    for (int w = 0; w < SDT_STAGE_BITS / 64; ++w) { t->mask[w] = mask[w]; t->recorded[w] = 0; }
    t->stride = 1;
    t->seen = 0;
    t->used = 0;
    t->slot = -1;
    for (int b = 0; b < SDT_STAGE_BITS; ++b)
        for (int k = 0; k < 2; ++k) t->ev[b][k] = nullptr;
    for (int b = 0; b < SDT_STAGE_BITS; ++b)
        for (int k = 0; k < 2; ++k) {
            if (!((mask[b >> 6] >> (b & 63)) & 1)) continue;
            t->ev[b][k] = new hipEvent_t[max_steps]();
            for (int i = 0; i < max_steps; ++i)
                if (hipEventCreate(&t->ev[b][k][i]) != hipSuccess) {
                    set_error("sdt_timing_create: hipEventCreate failed");
                    t->ev[b][k][i] = nullptr;
                    sdt_timing_destroy(t);
                    return SDT_ERR_HIP;
                }
        }
    *out = t;
    return SDT_OK;
}

extern "C" int32_t sdt_timing_create(int32_t max_steps, uint64_t stage_mask, sdt_timing** out) {
    const uint64_t mask[SDT_STAGE_BITS / 64] = {stage_mask, 0};
    return timing_create(max_steps, mask, out);
}

extern "C" int32_t sdt_timing_create_wide(int32_t max_steps, const uint64_t* stage_mask, sdt_timing** out) {
    return timing_create(max_steps, stage_mask, out);
}

extern "C" void sdt_timing_destroy(sdt_timing* t) {
    if (!t) return;
    for (int b = 0; b < SDT_STAGE_BITS; ++b)
        for (int k = 0; k < 2; ++k)
            if (t->ev[b][k]) {
                for (int i = 0; i < t->max_steps; ++i)
                    if (t->ev[b][k][i]) (void)hipEventDestroy(t->ev[b][k][i]);
                delete[] t->ev[b][k];
            }
    delete t;
}

extern "C" void sdt_timing_reset(sdt_timing* t) {
    if (t) {
        t->seen = 0; t->used = 0; t->slot = -1;
        for (int w = 0; w < SDT_STAGE_BITS / 64; ++w) t->recorded[w] = 0;
    }
}

extern "C" int32_t sdt_timing_set_stride(sdt_timing* t, int32_t stride) {
    SDT_REQUIRE(t && stride >= 1, SDT_ERR_INVALID_ARG, "sdt_timing_set_stride: null object or stride < 1");
    SDT_REQUIRE(t->seen == 0, SDT_ERR_INVALID_ARG, "sdt_timing_set_stride: set the stride before the first timed step (or after a reset)");
    t->stride = stride;
    return SDT_OK;
}

extern "C" int32_t sdt_timing_read(sdt_timing* t, int32_t kind, int32_t layer, float* ms_out, int32_t* n_out) {
    SDT_REQUIRE(t && ms_out && n_out && kind >= 0 && kind < SDT_STAGE_KINDS && layer >= 0 && layer < SDT_MAX_LAYERS,
                SDT_ERR_INVALID_ARG, "sdt_timing_read: bad arguments");
    const int bit = kind * SDT_MAX_LAYERS + layer;
    SDT_REQUIRE((t->mask[bit >> 6] >> (bit & 63)) & 1, SDT_ERR_INVALID_ARG, "sdt_timing_read: stage (%d,%d) was not selected", kind, layer);
    SDT_REQUIRE((t->recorded[bit >> 6] >> (bit & 63)) & 1, SDT_ERR_INVALID_ARG,
                "sdt_timing_read: stage (%d,%d) did not run as a separate stage", kind, layer);
    for (int i = 0; i < t->used; ++i) {
        if (hipEventSynchronize(t->ev[bit][1][i]) != hipSuccess ||
            hipEventElapsedTime(&ms_out[i], t->ev[bit][0][i], t->ev[bit][1][i]) != hipSuccess) {
            set_error("sdt_timing_read: event (%d,%d) of step slot %d was not recorded", kind, layer, i);
            return SDT_ERR_HIP;
        }
    }
    *n_out = t->used;
    return SDT_OK;
}

extern "C" int32_t sdt_train_step_layout(int64_t n_nodes, int32_t batch, const int32_t* fanouts, const sdt_model* model,
                                         int32_t dtype, sdt_step_layout* lay) {
    SDT_REQUIRE(lay, SDT_ERR_INVALID_ARG, "sdt_train_step_layout: null layout");
    int32_t rc = check_model(model, fanouts, "sdt_train_step_layout");
    if (rc != SDT_OK) return rc;
    SDT_REQUIRE(dtype_ok(dtype), SDT_ERR_INVALID_ARG, "sdt_train_step_layout: unknown dtype %d", dtype);
    SDT_REQUIRE(n_nodes >= 0 && n_nodes <= 0x7FFFFFFF && batch >= 0 && batch <= n_nodes, SDT_ERR_INVALID_ARG,
                "sdt_train_step_layout: n_nodes=%lld batch=%d", (long long)n_nodes, batch);
    const int L = model->n_layers;
    Caps c;
    SDT_REQUIRE(compute_caps(n_nodes, batch, fanouts, L, &c), SDT_ERR_INVALID_ARG,
                "sdt_train_step_layout: frontier bounds overflow int32");
    const size_t es = dtype_size(dtype);
    const int32_t* d = model->dims;
    *lay = sdt_step_layout{};
    lay->n_layers = L;
    Arena a(nullptr);
    size_t scratch = 0, bwd_scratch = 0;
    lay->header = a.take_off(64 * sizeof(int32_t));
    lay->state = a.take_off(sample_state_bytes(n_nodes));
    if (model->kind == SDT_MODEL_GAT) {
        for (int l = 0; l < L; ++l) {
            lay->cap_dst[l] = c.dst[l];
            lay->cap_src[l] = c.src[l];
            lay->cap_nnz[l] = c.nnz[l];
            lay->counts[l] = a.take_off(4 * sizeof(int32_t));
            lay->indptr[l] = a.take_off(((size_t)c.dst[l] + 1) * 4);
            lay->cols[l] = a.take_off((size_t)(c.nnz[l] > 0 ? c.nnz[l] : 1) * 4);
            lay->src_nodes[l] = a.take_off((size_t)(c.src[l] > 0 ? c.src[l] : 1) * 4);
            lay->t_indptr[l] = a.take_off(((size_t)c.src[l] + 1) * 4);
            lay->t_rows[l] = a.take_off((size_t)(c.nnz[l] > 0 ? c.nnz[l] : 1) * 4);
            if (l >= 1) lay->dH[l] = a.take_off((size_t)c.src[l] * d[l] * es);
            lay->H[l + 1] = a.take_off((size_t)c.dst[l] * d[l + 1] * (l == L - 1 ? 4 : es));
            lay->z[l] = a.take_off((size_t)c.src[l] * d[l + 1] * es);
            lay->dz[l] = a.take_off((size_t)c.src[l] * d[l + 1] * es);
            lay->dW[l] = a.take_off((size_t)d[l] * d[l + 1] * 4);
            lay->db[l] = a.take_off((size_t)d[l + 1] * 4);
            lay->datt[l] = a.take_off((size_t)2 * d[l + 1] * 4);
            lay->gatws[l] = a.take_off(sdt_gat_workspace_bytes(c.src[l], c.dst[l], d[l + 1]));
            Arena s(nullptr);
            size_t sb = sample_tmp_carve(s, n_nodes, c.dst[l], fanouts[l], nullptr);
            if (sb > scratch) scratch = sb;
            bwd_scratch += align_up(sdt_linear_bwd_workspace_bytes(c.src[l], d[l] / 2, d[l + 1]), 256);
        }
        if (bwd_scratch > scratch) scratch = bwd_scratch;
        lay->H[0] = a.take_off((size_t)c.src[0] * d[0] * es);
        lay->dZ = a.take_off((size_t)batch * d[L] * 4);
        lay->row_loss = a.take_off((size_t)(batch > 0 ? batch : 1) * 4);
        lay->scratch = a.take_off(scratch);
        lay->ld_in = (uint64_t)d[0];
        lay->total_bytes = a.off;
        return SDT_OK;
    }
    // GraphSAGE: input rows start on 128-byte lines (see sdt_step_layout::ld_in)
    const size_t line = 128 / es;
    const size_t ld0 = model->kind == SDT_MODEL_SAGE_MEAN ? ((size_t)d[0] + line - 1) / line * line : (size_t)d[0];
    lay->ld_in = ld0;
    for (int l = 0; l < L; ++l) {
        lay->cap_dst[l] = c.dst[l];
        lay->cap_src[l] = c.src[l];
        lay->cap_nnz[l] = c.nnz[l];
        lay->counts[l] = a.take_off(4 * sizeof(int32_t));
        lay->indptr[l] = a.take_off(((size_t)c.dst[l] + 1) * 4);
        lay->cols[l] = a.take_off((size_t)(c.nnz[l] > 0 ? c.nnz[l] : 1) * 4);
        lay->src_nodes[l] = a.take_off((size_t)(c.src[l] > 0 ? c.src[l] : 1) * 4);
        if (l >= 1) {
            lay->t_indptr[l] = a.take_off(((size_t)c.src[l] + 1) * 4);
            lay->t_rows[l] = a.take_off((size_t)(c.nnz[l] > 0 ? c.nnz[l] : 1) * 4);
            lay->dH[l] = a.take_off((size_t)c.src[l] * d[l] * es);
            lay->dSelf[l] = a.take_off((size_t)c.dst[l] * d[l] * es);
            lay->dAgg[l] = a.take_off((size_t)c.dst[l] * d[l] * es);
        }
        lay->A[l] = a.take_off((size_t)c.dst[l] * (l == 0 ? ld0 : (size_t)d[l]) * es);
        lay->H[l + 1] = a.take_off((size_t)c.dst[l] * d[l + 1] * (l == L - 1 ? 4 : es));
        lay->dW[l] = a.take_off((size_t)2 * d[l] * d[l + 1] * 4);
        lay->db[l] = a.take_off((size_t)d[l + 1] * 4);
        Arena s(nullptr);
        size_t sb = sample_tmp_carve(s, n_nodes, c.dst[l], fanouts[l], nullptr);
        if (sb > scratch) scratch = sb;
        bwd_scratch += bwd_scratch_bytes(batch, c.dst[l], operand_width(model, l), d[l + 1], l == L - 1);
    }
    // the sampling scratch is dead once phase 2 starts; the backward keeps one region per layer
    // alive until the single reduction launch at the end of the step
    if (bwd_scratch > scratch) scratch = bwd_scratch;
    lay->H[0] = a.take_off((size_t)c.dst[0] * ld0 * es);
    lay->dZ = a.take_off((size_t)batch * d[L] * 4);
    lay->row_loss = a.take_off((size_t)(batch > 0 ? batch : 1) * 4);
    lay->scratch = a.take_off(scratch);
    if (dtype == SDT_BF16) {
        size_t wb = 0;
        for (int l = 0; l < L; ++l) wb += bf16_weights_bytes(d[l], d[l + 1]);
        lay->wlow = a.take_off(wb);
    } else if (model->kind == SDT_MODEL_SAGE_MEAN) {
        // transposed weights of the layers whose forward runs on split-bf16 (kept across the steps of a loop)
        size_t wb = 0;
        for (int l = 0; l + 1 < L; ++l)
            if (x3_fwd_wanted(c.dst[l], d[l], d[l + 1])) wb += x3_fwd_image_bytes(d[l], d[l + 1]);
        if (wb > 0) lay->wlow = a.take_off(wb);
    }
    if (model->kind == SDT_MODEL_GCN)
        for (int l = 0; l < L; ++l)
            lay->norm[l] = a.take_off(align_up((size_t)(c.src[l] > 0 ? c.src[l] : 1) * 4, 256) +
                                      2 * align_up((size_t)(c.dst[l] > 0 ? c.dst[l] : 1) * 4, 256));
    lay->total_bytes = a.off;
    return SDT_OK;
}

namespace {

// Everything one step needs, resolved once per call.
// SGD or Adam, from the model struct; `step` is the 0-based update counter
OptArgs optimizer_args(const sdt_model* m, float lr, uint32_t step) {
    OptArgs o;
    o.lr = lr;
    if (m->optimizer == SDT_OPT_ADAM) {
        o.adam = 1;
        o.beta1 = m->beta1;
        o.beta2 = m->beta2;
        o.eps = m->eps;
        const double t = (double)step + 1.0;
        o.c1 = (float)(1.0 / (1.0 - pow((double)m->beta1, t)));
        o.c2 = (float)(1.0 / (1.0 - pow((double)m->beta2, t)));
    }
    return o;
}
// Adam moments of a layer's (W, b) reduction
void attach_moments(PendingReduce* pr, const sdt_model* m, int l) {
    if (m->optimizer != SDT_OPT_ADAM) return;
    pr->mW = m->mW[l];
    pr->vW = m->vW[l];
    pr->mb = m->mb[l];
    pr->vb = m->vb[l];
}

struct StepCtx {
    const sdt_csr* graph;
    const void* X;
    int64_t ldx;
    int32_t dtype;
    const int32_t* labels;
    int32_t batch;
    const int32_t* fanouts;
    const sdt_model* model;
    uint64_t seed;
    float lr;
    sdt_timing* timing;
    sdt_step_layout lay;
    int32_t slot = -1;   // timing slot of the step being enqueued (each enqueueing thread has its own copy)
    // Inside a loop call the images of the weights that the matrix-core paths read (bf16 images, transposed fp32
    // weights) live in ONE place for all steps -- the model side of the steps runs in sequence on one stream -- and
    // every update launch rewrites them with the weights; only the call's first step builds them from the weights.
    // Null: a step on its own, which builds them in its own workspace every time.
    char* images = nullptr;
    bool images_current = false;
};

struct StepBuffers {
    char* base;
    size_t bytes;
    sdt_block blk[SDT_MAX_LAYERS];
    void* at(uint64_t off) const { return base + off; }
    // GCN normalisation vectors of layer l (see sdt_step_layout::norm)
    float* gcn_c(const sdt_step_layout& lay, int l) const { return static_cast<float*>(at(lay.norm[l])); }
    float* gcn_s(const sdt_step_layout& lay, int l) const {
        return reinterpret_cast<float*>(base + lay.norm[l] + align_up((size_t)(lay.cap_src[l] > 0 ? lay.cap_src[l] : 1) * 4, 256));
    }
    float* gcn_self(const sdt_step_layout& lay, int l) const {
        return reinterpret_cast<float*>(reinterpret_cast<char*>(gcn_s(lay, l)) +
                                        align_up((size_t)(lay.cap_dst[l] > 0 ? lay.cap_dst[l] : 1) * 4, 256));
    }
};

int32_t check_step_args(const char* who, const sdt_csr* graph, const void* X, int64_t ldx, const int32_t* labels,
                        const int32_t* seeds, int32_t batch, const sdt_model* model, const float* loss_d) {
    SDT_REQUIRE(batch > 0, SDT_ERR_INVALID_ARG, "%s: empty batch", who);
    SDT_REQUIRE(X && labels && seeds && loss_d && ldx >= model->dims[0], SDT_ERR_INVALID_ARG,
                "%s: null input or ldx < dims[0]", who);
    SDT_REQUIRE(graph->indices || graph->n_nodes == 0, SDT_ERR_INVALID_ARG, "%s: null indices", who);
    for (int l = 0; l < model->n_layers; ++l)
        SDT_REQUIRE(model->W[l] && model->b[l], SDT_ERR_INVALID_ARG, "%s: null weights of layer %d", who, l);
    SDT_REQUIRE(model->optimizer == SDT_OPT_SGD || model->optimizer == SDT_OPT_ADAM, SDT_ERR_INVALID_ARG,
                "%s: unknown optimizer %d", who, model->optimizer);
    if (model->optimizer == SDT_OPT_ADAM) {
        SDT_REQUIRE(model->beta1 >= 0.f && model->beta1 < 1.f && model->beta2 >= 0.f && model->beta2 < 1.f && model->eps > 0.f,
                    SDT_ERR_INVALID_ARG, "%s: Adam needs 0 <= beta < 1 and eps > 0", who);
        for (int l = 0; l < model->n_layers; ++l)
            SDT_REQUIRE(model->mW[l] && model->vW[l] && model->mb[l] && model->vb[l] &&
                            (model->kind != SDT_MODEL_GAT || (model->matt[l] && model->vatt[l])),
                        SDT_ERR_INVALID_ARG, "%s: Adam needs the moment buffers of layer %d", who, l);
    }
    if (model->kind == SDT_MODEL_GAT)
        for (int l = 0; l < model->n_layers; ++l)
            SDT_REQUIRE(model->att[l], SDT_ERR_INVALID_ARG, "%s: null attention vectors of layer %d", who, l);
    return SDT_OK;
}

void bind_buffers(const sdt_step_layout& lay, void* ws, size_t bytes, StepBuffers* b) {
    b->base = static_cast<char*>(ws);
    b->bytes = bytes;
    for (int l = 0; l < lay.n_layers; ++l) {
        sdt_block& k = b->blk[l];
        k.cap_dst = lay.cap_dst[l];
        k.cap_src = lay.cap_src[l];
        k.cap_nnz = lay.cap_nnz[l];
        k.reserved = 0;
        k.counts = static_cast<int32_t*>(b->at(lay.counts[l]));
        k.indptr = static_cast<int32_t*>(b->at(lay.indptr[l]));
        k.cols = static_cast<int32_t*>(b->at(lay.cols[l]));
        k.src_nodes = static_cast<int32_t*>(b->at(lay.src_nodes[l]));
        // the transposed block exists where an input gradient flows through the block (offset 0 = absent)
        k.t_indptr = lay.t_indptr[l] ? static_cast<int32_t*>(b->at(lay.t_indptr[l])) : nullptr;
        k.t_rows = lay.t_rows[l] ? static_cast<int32_t*>(b->at(lay.t_rows[l])) : nullptr;
    }
}

// Phase 1 (needs no weights): sample from the seeds outwards, then gather the input features
// of the outermost frontier.  The frontier state (two bits per node, the node -> local-id map)
// carries over from layer to layer and is rebuilt from nothing by every step.
int32_t step_sample(const StepCtx& c, const StepBuffers& b, const int32_t* seeds, uint32_t step, hipStream_t st) {
    const sdt_step_layout& lay = c.lay;
    const int L = c.model->n_layers;
    const int32_t* d = c.model->dims;
    const int64_t N = c.graph->n_nodes;
    SampleWs sw{};
    sample_state_carve(b.at(lay.state), N, &sw);
    int32_t rc;
    const int32_t* dst = seeds;
    const int32_t* n_d = nullptr;
    for (int l = L - 1; l >= 0; --l) {
        StageTimer tl(c.timing, c.slot, SDT_STAGE_SAMPLE, l, st);
        if (l == L - 1) {
            // every step starts from an empty frontier: the state words are cleared, whatever the
            // workspace held (nothing in it is carried from step to step), then the seeds join
            rc = sample_state_clear(sw, N, st);
            if (rc != SDT_OK) return rc;
            rc = sample_seed_map(sw, seeds, c.batch, nullptr, st);
            if (rc != SDT_OK) return rc;
        }
        Arena a(b.at(lay.scratch));
        sample_tmp_carve(a, N, lay.cap_dst[l], c.fanouts[l], &sw);
        // the nodes a layer adds are looked up in the map only by the layers sampled after it
        rc = sample_layer(*c.graph, dst, lay.cap_dst[l], n_d, c.fanouts[l], c.seed, step, (uint32_t)l, b.blk[l], sw,
                          /*write_map=*/l > 0, st, c.timing, c.slot);
        if (rc != SDT_OK) return rc;
        dst = b.blk[l].src_nodes;
        n_d = b.blk[l].counts + 1;
    }
    if (c.model->kind == SDT_MODEL_GCN) {
        // normalisation vectors of every block, then layer 0's aggregation straight out of X
        for (int l = 0; l < L; ++l) {
            rc = sdt_gcn_norm(c.graph, &b.blk[l], b.gcn_c(lay, l), b.gcn_s(lay, l), b.gcn_self(lay, l), st);
            if (rc != SDT_OK) return rc;
        }
        SDT_REQUIRE(lay.cap_dst[0] == 0 || aligned16(c.X), SDT_ERR_INVALID_ARG, "sdt_train_step: X must be 16-byte aligned");
        StageTimer tm(c.timing, c.slot, SDT_STAGE_AGG_FWD, 0, st);
        return gcn_aggregate_fwd(&b.blk[0], c.X, c.ldx, true, d[0], c.dtype, b.gcn_c(lay, 0), b.gcn_s(lay, 0),
                                 b.gcn_self(lay, 0), b.at(lay.A[0]), d[0], st);
    }
    if (c.model->kind == SDT_MODEL_GAT) {
        // every frontier row is projected, so every one is gathered
        StageTimer tm(c.timing, c.slot, SDT_STAGE_GATHER, 0, st);
        return gather_rows(c.X, c.ldx, d[0], c.dtype, b.blk[0].src_nodes, lay.cap_src[0], b.blk[0].counts + 1, b.at(lay.H[0]),
                           d[0], false, nullptr, st);
    }
    // Input features: only the destination prefix of the outermost frontier is copied (the
    // projection's "self" operand); the neighbour mean of layer 0 is taken straight out of X.
    // The copy also zeroes the row padding of H[0] and of A[0] (same rows, same stride).
    {
        StageTimer tm(c.timing, c.slot, SDT_STAGE_GATHER, 0, st);
        rc = gather_rows(c.X, c.ldx, d[0], c.dtype, b.blk[0].src_nodes, lay.cap_dst[0], b.blk[0].counts,
                         b.at(lay.H[0]), (int64_t)lay.ld_in, /*zero_pad=*/true, /*also_pad=*/b.at(lay.A[0]), st);
    }
    if (rc != SDT_OK) return rc;
    StageTimer tm(c.timing, c.slot, SDT_STAGE_AGG_FWD, 0, st);
    return aggregate_gather_fwd(&b.blk[0], c.X, c.ldx, d[0], c.dtype, b.at(lay.A[0]), (int64_t)lay.ld_in, st);
}

// Phase 2 of a GCN step.  The projection kernels take two operands of equal width; here they are
// the two halves of the aggregated row, so W[l] = [in, out] is exactly their [2 * in/2, out] weight
// and their two input gradients land side by side as the gradient w.r.t. the aggregated row.
int32_t step_compute_gcn(const StepCtx& c, const StepBuffers& b, const int32_t* seeds, uint32_t step, float* loss_d,
                         hipStream_t st) {
    const sdt_step_layout& lay = c.lay;
    const sdt_model* model = c.model;
    const int L = model->n_layers;
    const int32_t* d = model->dims;
    sdt_timing* timing = c.timing;
    const int32_t dtype = c.dtype;
    const size_t es = dtype_size(dtype);
    int32_t rc;
    const int hl = d[L - 1] / 2;
    const bool fused_head = head_supported(hl, d[L]) && aligned16(model->W[L - 1]);
    size_t scr_off[SDT_MAX_LAYERS], scr_len[SDT_MAX_LAYERS];
    {
        size_t o = lay.scratch;
        for (int l = 0; l < L; ++l) {
            scr_len[l] = bwd_scratch_bytes(c.batch, lay.cap_dst[l], d[l] / 2, d[l + 1], l == L - 1);
            scr_off[l] = o;
            o += scr_len[l];
        }
    }
    PendingReduce pending[SDT_MAX_LAYERS];
    int n_pending = 0;
    // bf16 storage: the products take the operands widened on the way into LDS and the weights rounded to bf16
    // where they enter (the general kernels; the bf16 weight images of the GraphSAGE kind have another shape)
    auto half0 = [&](int l) { return static_cast<char*>(b.at(lay.A[l])); };
    auto half1 = [&](int l) { return static_cast<char*>(b.at(lay.A[l])) + (size_t)(d[l] / 2) * es; };
    for (int l = 0; l < L; ++l) {
        if (l > 0) {
            StageTimer tm(timing, c.slot, SDT_STAGE_AGG_FWD, l, st);
            rc = sdt_gcn_aggregate_fwd(&b.blk[l], b.at(lay.H[l]), d[l], 0, d[l], dtype, b.gcn_c(lay, l), b.gcn_s(lay, l),
                                       b.gcn_self(lay, l), b.at(lay.A[l]), d[l], st);
            if (rc != SDT_OK) return rc;
        }
        const bool last = l == L - 1;
        if (last && fused_head) break;
        StageTimer tm(timing, c.slot, SDT_STAGE_LINEAR_FWD, l, st);
        rc = linear_fwd(half0(l), d[l], half1(l), d[l], lay.cap_dst[l], b.blk[l].counts, d[l] / 2, d[l + 1], model->W[l],
                        model->b[l], last ? 0 : 1, dtype, b.at(lay.H[l + 1]), d[l + 1], last ? SDT_F32 : dtype,
                        /*rows_padded=*/false, st);
        if (rc != SDT_OK) return rc;
    }
    if (!fused_head) {
        StageTimer tm(timing, c.slot, SDT_STAGE_LOSS, 0, st);
        rc = softmax_xent(static_cast<const float*>(b.at(lay.H[L])), d[L], c.batch, d[L], c.labels, seeds,
                          static_cast<float*>(b.at(lay.dZ)), static_cast<float*>(b.at(lay.row_loss)), st);
        if (rc != SDT_OK) return rc;
    }
    const void* dY = b.at(lay.dZ);
    int32_t dy_dtype = SDT_F32;
    for (int l = L - 1; l >= 0; --l) {
        float* dW = model->dW[l] ? model->dW[l] : static_cast<float*>(b.at(lay.dW[l]));
        float* db = model->db[l] ? model->db[l] : static_cast<float*>(b.at(lay.db[l]));
        const bool inner = l > 0;
        char* dA = inner ? static_cast<char*>(b.at(lay.dAgg[l])) : nullptr;   // gradient w.r.t. the aggregated row
        BwdExtras ex;
        ex.defer = &pending[n_pending++];
        ex.W_upd = model->W[l];
        ex.b_upd = model->b[l];
        {
            StageTimer tm(timing, c.slot, SDT_STAGE_LINEAR_BWD, l, st);
            if (l == L - 1 && fused_head) {
                float *P, *Q;
                {
                    StageTimer th(timing, c.slot, SDT_STAGE_HEAD, l, st);
                    rc = head_fwd_bwd(half0(l), d[l], half1(l), d[l], c.batch, hl, d[l + 1], model->W[l], model->b[l], dtype,
                                      c.labels, seeds, static_cast<float*>(b.at(lay.H[L])), static_cast<float*>(b.at(lay.dZ)),
                                      static_cast<float*>(b.at(lay.row_loss)), dA, inner ? dA + (size_t)hl * es : nullptr, d[l],
                                      b.at(scr_off[l]), scr_len[l], &P, &Q, st);
                }
                if (rc != SDT_OK) return rc;
                rc = reduce_partials(P, Q, head_splits(c.batch), hl, d[l + 1], dW, db, ex, st);
            } else {
                rc = linear_bwd(dY, d[l + 1], dy_dtype, nullptr, 0, 0, half0(l), d[l], half1(l), d[l], lay.cap_dst[l],
                                b.blk[l].counts, d[l] / 2, d[l + 1], model->W[l], dtype, dW, db, dA,
                                inner ? dA + (size_t)(d[l] / 2) * es : nullptr, d[l], b.at(scr_off[l]), scr_len[l], ex, st);
            }
            if (rc != SDT_OK) return rc;
        }
        if (inner) {
            StageTimer tm(timing, c.slot, SDT_STAGE_AGG_BWD, l, st);
            rc = sdt_gcn_aggregate_bwd(&b.blk[l], dA, d[l], b.at(lay.H[l]), d[l], dtype, b.gcn_c(lay, l), b.gcn_s(lay, l),
                                       b.gcn_self(lay, l), b.at(lay.dH[l]), d[l], st);
            if (rc != SDT_OK) return rc;
            dY = b.at(lay.dH[l]);
            dy_dtype = dtype;
        }
    }
    for (int k = 0; k < n_pending; ++k) attach_moments(&pending[k], model, L - 1 - k);   // queued last layer first
    StageTimer tu(timing, c.slot, SDT_STAGE_UPDATE, 0, st);
    return reduce_all(pending, n_pending, optimizer_args(model, c.lr, step), static_cast<const float*>(b.at(lay.row_loss)),
                      c.batch, loss_d, st);
}

// Phase 2 of a GAT step.  The projection z = H W covers every frontier row (the attention needs the
// projected neighbours) and runs on the GraphSAGE kernels with the two halves of a row as operands;
// the bias is added after the aggregation, so its gradient (column sums of the masked output
// gradient) and the attention vectors' are summed by the step's single reduction launch from
// per-chunk partials: the former replaces the projection kernels' own column sums, the latter is
// queued as a second reduction of the layer with no weight part.
int32_t step_compute_gat(const StepCtx& c, const StepBuffers& b, const int32_t* seeds, uint32_t step, float* loss_d,
                         hipStream_t st) {
    const sdt_step_layout& lay = c.lay;
    const sdt_model* model = c.model;
    const int L = model->n_layers;
    const int32_t* d = model->dims;
    sdt_timing* timing = c.timing;
    const float slope = model->gat_slope;
    const int32_t dtype = c.dtype;
    const size_t es = dtype_size(dtype);
    int32_t rc;
    size_t scr_off[SDT_MAX_LAYERS], scr_len[SDT_MAX_LAYERS], gws_len[SDT_MAX_LAYERS];
    {
        size_t o = lay.scratch;
        for (int l = 0; l < L; ++l) {
            scr_len[l] = align_up(sdt_linear_bwd_workspace_bytes(lay.cap_src[l], d[l] / 2, d[l + 1]), 256);
            scr_off[l] = o;
            o += scr_len[l];
            gws_len[l] = sdt_gat_workspace_bytes(lay.cap_src[l], lay.cap_dst[l], d[l + 1]);
        }
    }
    // bf16 storage: the gathered rows, the projected rows z, the hidden activations and the gradients w.r.t. all three
    // are bf16 (rounded when stored); the logits, the loss gradient, the attention scalars and every sum stay fp32
    auto H = [&](int l) { return static_cast<char*>(b.at(lay.H[l])); };
    auto H1 = [&](int l) { return static_cast<char*>(b.at(lay.H[l])) + (size_t)(d[l] / 2) * es; };
    auto Z = [&](int l) { return b.at(lay.z[l]); };
    for (int l = 0; l < L; ++l) {
        const int F = d[l + 1];
        {
            StageTimer tm(timing, c.slot, SDT_STAGE_LINEAR_FWD, l, st);
            rc = linear_fwd(H(l), d[l], H1(l), d[l], lay.cap_src[l], b.blk[l].counts + 1, d[l] / 2, F, model->W[l], nullptr, 0,
                            dtype, Z(l), F, dtype, /*rows_padded=*/false, st);
            if (rc != SDT_OK) return rc;
        }
        StageTimer tm(timing, c.slot, SDT_STAGE_AGG_FWD, l, st);
        rc = gat_forward(&b.blk[l], Z(l), F, F, dtype, model->att[l], model->att[l] + F, slope, model->b[l], l < L - 1 ? 1 : 0,
                         H(l + 1), F, l < L - 1 ? dtype : SDT_F32, b.at(lay.gatws[l]), gws_len[l], st);
        if (rc != SDT_OK) return rc;
    }
    {
        StageTimer tm(timing, c.slot, SDT_STAGE_LOSS, 0, st);
        rc = softmax_xent(static_cast<const float*>(b.at(lay.H[L])), d[L], c.batch, d[L], c.labels, seeds,
                          static_cast<float*>(b.at(lay.dZ)), static_cast<float*>(b.at(lay.row_loss)), st);
        if (rc != SDT_OK) return rc;
    }
    PendingReduce pending[2 * SDT_MAX_LAYERS];
    int n_pending = 0;
    void* g = b.at(lay.dZ);
    int32_t g_dtype = SDT_F32;
    for (int l = L - 1; l >= 0; --l) {
        const int F = d[l + 1];
        float* dW = model->dW[l] ? model->dW[l] : static_cast<float*>(b.at(lay.dW[l]));
        float* db = model->db[l] ? model->db[l] : static_cast<float*>(b.at(lay.db[l]));
        float* datt = model->datt[l] ? model->datt[l] : static_cast<float*>(b.at(lay.datt[l]));
        void* dz = b.at(lay.dz[l]);
        const bool inner = l > 0;
        const float *Qb, *part;
        int32_t n_chunks, n_part;
        {
            StageTimer tm(timing, c.slot, SDT_STAGE_AGG_BWD, l, st);
            // g: gradient w.r.t. this layer's output; masked in place by the layer's own ReLU (not the last layer)
            rc = gat_mask_bias(&b.blk[l], g, F, l < L - 1 ? H(l + 1) : nullptr, F, F, g_dtype, b.at(lay.gatws[l]), gws_len[l],
                               &Qb, &n_chunks, st);
            if (rc != SDT_OK) return rc;
            rc = gat_backward(&b.blk[l], Z(l), F, F, dtype, model->att[l], model->att[l] + F, slope, g, F, g_dtype, dz, F,
                              b.at(lay.gatws[l]), gws_len[l], &part, &n_part, st);
            if (rc != SDT_OK) return rc;
        }
        PendingReduce* pw = &pending[n_pending++];
        {
            StageTimer tm(timing, c.slot, SDT_STAGE_LINEAR_BWD, l, st);
            BwdExtras ex;
            ex.defer = pw;
            ex.W_upd = model->W[l];
            char* dH = inner ? static_cast<char*>(b.at(lay.dH[l])) : nullptr;
            rc = linear_bwd(dz, F, dtype, nullptr, 0, 0, H(l), d[l], H1(l), d[l], lay.cap_src[l], b.blk[l].counts + 1, d[l] / 2, F,
                            model->W[l], dtype, dW, db, dH, inner ? dH + (size_t)(d[l] / 2) * es : nullptr, d[l],
                            b.at(scr_off[l]), scr_len[l], ex, st);
            if (rc != SDT_OK) return rc;
            g = dH;
            g_dtype = dtype;
        }
        // the bias gradient is the column sum of the masked output gradient, not of dz
        pw->Q = Qb;
        pw->q_splits = n_chunks;
        pw->q_rows_d = b.blk[l].counts;          // n_dst
        pw->q_chunk_rows = GAT_CHUNK_ROWS;
        pw->db = db;
        pw->b_upd = model->b[l];
        attach_moments(pw, model, l);
        PendingReduce* pa = &pending[n_pending++];
        pa->Q = part;
        pa->q_splits = n_part;
        pa->q_rows_d = b.blk[l].counts + 1;      // n_src
        pa->q_chunk_rows = GAT_CHUNK_ROWS;
        pa->in = 0;
        pa->out = 2 * F;
        pa->db = datt;
        pa->b_upd = model->att[l];
        if (model->optimizer == SDT_OPT_ADAM) {
            pa->mb = model->matt[l];
            pa->vb = model->vatt[l];
        }
    }
    StageTimer tu(timing, c.slot, SDT_STAGE_UPDATE, 0, st);
    return reduce_all(pending, n_pending, optimizer_args(model, c.lr, step), static_cast<const float*>(b.at(lay.row_loss)),
                      c.batch, loss_d, st);
}

// Phase 2: forward, loss, backward, SGD on the blocks and features phase 1 left in `b`.
// `step` is the update counter (Adam's bias correction uses step + 1).
int32_t step_compute(const StepCtx& c, const StepBuffers& b, const int32_t* seeds, uint32_t step, float* loss_d,
                     hipStream_t st) {
    if (c.model->kind == SDT_MODEL_GCN) return step_compute_gcn(c, b, seeds, step, loss_d, st);
    if (c.model->kind == SDT_MODEL_GAT) return step_compute_gat(c, b, seeds, step, loss_d, st);
    const sdt_step_layout& lay = c.lay;
    const sdt_model* model = c.model;
    const int L = model->n_layers;
    const int32_t* d = model->dims;
    const int32_t dtype = c.dtype;
    sdt_timing* timing = c.timing;
    int32_t rc;
    // Small class counts: the last layer's projection, the loss and that layer's backward run
    // as one fused launch (head.hip) instead of five.
    const bool fused_head = head_supported(d[L - 1], d[L]) && aligned16(model->W[L - 1]);
    // one scratch region per layer, laid end to end (see sdt_train_step_layout)
    size_t scr_off[SDT_MAX_LAYERS], scr_len[SDT_MAX_LAYERS];
    {
        size_t o = lay.scratch;
        for (int l = 0; l < L; ++l) {
            scr_len[l] = bwd_scratch_bytes(c.batch, lay.cap_dst[l], d[l], d[l + 1], l == L - 1);
            scr_off[l] = o;
            o += scr_len[l];
        }
    }
    PendingReduce pending[SDT_MAX_LAYERS];
    int n_pending = 0;
    // row stride of H[l] and A[l]: the input rows are padded to whole 128-byte lines, readable to the stride
    auto ldx = [&](int l) { return l == 0 ? (int64_t)lay.ld_in : (int64_t)d[l]; };
    // bf16 activations: the matrix products run on the bf16 matrix cores from bf16 images of the
    // weights, rewritten here every step (the weights are the caller's and change every step)
    char* wt[SDT_MAX_LAYERS] = {};
    char* wb[SDT_MAX_LAYERS] = {};
    float* wx3[SDT_MAX_LAYERS] = {};   // fp32: transposed weights of the split-bf16 forward, kept across a loop's steps
    char* const images = c.images ? c.images : static_cast<char*>(b.at(lay.wlow));
    const bool images_current = c.images && c.images_current;
    if (dtype == SDT_BF16) {
        if (!images_current) {
            rc = convert_weights_bf16(model, images, st);
            if (rc != SDT_OK) return rc;
        }
        char* p = images;
        for (int l = 0; l < L; ++l) {
            wt[l] = p;
            wb[l] = p + align_up((size_t)2 * d[l] * d[l + 1] * 2, 256);
            p += bf16_weights_bytes(d[l], d[l + 1]);
        }
    } else if (c.images) {
        char* p = images;
        for (int l = 0; l + 1 < L; ++l)
            if (x3_fwd_wanted(lay.cap_dst[l], d[l], d[l + 1])) {
                wx3[l] = reinterpret_cast<float*>(p);
                p += x3_fwd_image_bytes(d[l], d[l + 1]);
            }
    }
    for (int l = 0; l < L; ++l) {
        if (l > 0) {   // layer 0's mean was taken in phase 1
            StageTimer tm(timing, c.slot, SDT_STAGE_AGG_FWD, l, st);
            rc = sdt_sage_aggregate_fwd(&b.blk[l], b.at(lay.H[l]), d[l], d[l], dtype, b.at(lay.A[l]), d[l], st);
            if (rc != SDT_OK) return rc;
        }
        const bool last = l == L - 1;
        if (last && fused_head) break;
        StageTimer tm(timing, c.slot, SDT_STAGE_LINEAR_FWD, l, st);
        if (dtype == SDT_BF16 && bf16_mfma_fwd_ok(b.at(lay.H[l]), ldx(l), b.at(lay.A[l]), ldx(l), d[l]))
            rc = linear_fwd_bf16(b.at(lay.H[l]), ldx(l), b.at(lay.A[l]), ldx(l), lay.cap_dst[l], b.blk[l].counts, d[l],
                                 d[l + 1], wt[l], model->b[l], last ? 0 : 1, b.at(lay.H[l + 1]), d[l + 1],
                                 last ? SDT_F32 : dtype, st);
        else if (dtype == SDT_F32 && !last && x3_fwd_wanted(lay.cap_dst[l], d[l], d[l + 1]) &&
                 x3_fwd_ok(b.at(lay.H[l]), ldx(l), b.at(lay.A[l]), ldx(l), d[l], /*rows_padded=*/l == 0, b.at(lay.H[l + 1]),
                           d[l + 1]))
            // few row tiles, wide output, long reduction: exact bf16 triple splits on the bf16 matrix cores; the
            // layer's backward scratch is free until the backward reaches this layer
            rc = linear_fwd_x3(static_cast<const float*>(b.at(lay.H[l])), ldx(l), static_cast<const float*>(b.at(lay.A[l])),
                               ldx(l), lay.cap_dst[l], b.blk[l].counts, d[l], d[l + 1], model->W[l], model->b[l], 1,
                               static_cast<float*>(b.at(lay.H[l + 1])), d[l + 1], b.at(scr_off[l]), scr_len[l], wx3[l],
                               images_current, st);
        else
            rc = linear_fwd(b.at(lay.H[l]), ldx(l), b.at(lay.A[l]), ldx(l), lay.cap_dst[l], b.blk[l].counts, d[l],
                            d[l + 1], model->W[l], model->b[l], last ? 0 : 1, dtype, b.at(lay.H[l + 1]),
                            d[l + 1], last ? SDT_F32 : dtype, /*rows_padded=*/l == 0, st);
        if (rc != SDT_OK) return rc;
    }
    if (!fused_head) {
        StageTimer tm(timing, c.slot, SDT_STAGE_LOSS, 0, st);
        rc = softmax_xent(static_cast<const float*>(b.at(lay.H[L])), d[L], c.batch, d[L], c.labels, seeds,
                          static_cast<float*>(b.at(lay.dZ)), static_cast<float*>(b.at(lay.row_loss)), st);
        if (rc != SDT_OK) return rc;
    }
    const void* dY = b.at(lay.dZ);
    int32_t dy_dtype = SDT_F32;
    for (int l = L - 1; l >= 0; --l) {
        float* dW = model->dW[l] ? model->dW[l] : static_cast<float*>(b.at(lay.dW[l]));
        float* db = model->db[l] ? model->db[l] : static_cast<float*>(b.at(lay.db[l]));
        const bool inner = l > 0;
        if (l == L - 1 && fused_head) {
            StageTimer tm(timing, c.slot, SDT_STAGE_LINEAR_BWD, l, st);
            float *P, *Q;
            {
            StageTimer th(timing, c.slot, SDT_STAGE_HEAD, l, st);
            rc = head_fwd_bwd(b.at(lay.H[l]), ldx(l), b.at(lay.A[l]), ldx(l), c.batch, d[l], d[l + 1], model->W[l],
                              model->b[l], dtype, c.labels, seeds, static_cast<float*>(b.at(lay.H[L])),
                              static_cast<float*>(b.at(lay.dZ)), static_cast<float*>(b.at(lay.row_loss)),
                              inner ? b.at(lay.dSelf[l]) : nullptr, inner ? b.at(lay.dAgg[l]) : nullptr, d[l],
                              b.at(scr_off[l]), scr_len[l], &P, &Q, st);
            }
            if (rc != SDT_OK) return rc;
            BwdExtras ex;
            ex.defer = &pending[n_pending++];
            ex.W_upd = model->W[l];
            ex.b_upd = model->b[l];
            rc = reduce_partials(P, Q, head_splits(c.batch), d[l], d[l + 1], dW, db, ex, st);
            if (rc != SDT_OK) return rc;
        } else {
            StageTimer tm(timing, c.slot, SDT_STAGE_LINEAR_BWD, l, st);
            BwdExtras ex;
            ex.defer = &pending[n_pending++];
            ex.Wb = wb[l];
            ex.W_upd = model->W[l];
            ex.b_upd = model->b[l];
            ex.rows_padded = l == 0;
            ex.x3 = true;
            ex.timing = timing; ex.slot = c.slot; ex.layer = l;
            rc = linear_bwd(dY, d[l + 1], dy_dtype, nullptr, 0, 0, b.at(lay.H[l]), ldx(l), b.at(lay.A[l]), ldx(l),
                            lay.cap_dst[l], b.blk[l].counts, d[l], d[l + 1], model->W[l], dtype, dW, db,
                            inner ? b.at(lay.dSelf[l]) : nullptr, inner ? b.at(lay.dAgg[l]) : nullptr, d[l],
                            b.at(scr_off[l]), scr_len[l], ex, st);
            if (rc != SDT_OK) return rc;
        }
        if (inner) {
            // gradient w.r.t. H[l], masked by the ReLU that produced H[l]
            StageTimer tm(timing, c.slot, SDT_STAGE_AGG_BWD, l, st);
            rc = sdt_sage_aggregate_bwd(&b.blk[l], b.at(lay.dAgg[l]), d[l], b.at(lay.dSelf[l]), d[l], b.at(lay.H[l]), d[l],
                                        dtype, b.at(lay.dH[l]), d[l], st);
            if (rc != SDT_OK) return rc;
            dY = b.at(lay.dH[l]);
            dy_dtype = dtype;
        }
    }
    // One launch finishes every layer: the split partial products of all weight gradients are
    // summed in a fixed order, the SGD step is applied, and the per-seed losses are averaged.
    // (No layer's weights were touched before this point, so every product above saw the
    // weights the step started with.)
    for (int k = 0; k < n_pending; ++k) {   // queued last layer first
        const int l = L - 1 - k;
        attach_moments(&pending[k], model, l);
        if (c.images) {   // the next step of the loop reads the images this update leaves
            if (dtype == SDT_BF16) {
                pending[k].img_wt = reinterpret_cast<uint16_t*>(wt[l]);
                pending[k].img_wb = reinterpret_cast<uint16_t*>(wb[l]);
                pending[k].img_ldb = bf16_ldb(d[l + 1]);
            } else if (wx3[l]) {
                pending[k].img_x3 = wx3[l];
                pending[k].img_kp = x3_fwd_image_kp(d[l]);
            }
        }
    }
    StageTimer tu(timing, c.slot, SDT_STAGE_UPDATE, 0, st);
    return reduce_all(pending, n_pending, optimizer_args(model, c.lr, step), static_cast<const float*>(b.at(lay.row_loss)),
                      c.batch, loss_d, st);
}

}  // namespace

extern "C" int32_t sdt_train_step(const sdt_csr* graph, const void* X, int64_t ldx, int32_t dtype, const int32_t* labels,
                                  const int32_t* seeds, int32_t batch, const int32_t* fanouts, const sdt_model* model,
                                  uint64_t seed, uint32_t step, float lr, float* loss_d, sdt_timing* timing, void* ws,
                                  size_t ws_bytes, void* stream) {
    SDT_REQUIRE(graph && graph->indptr, SDT_ERR_INVALID_ARG, "sdt_train_step: null graph");
    StepCtx c{graph, X, ldx, dtype, labels, batch, fanouts, model, seed, lr, timing, {}};
    int32_t rc = sdt_train_step_layout(graph->n_nodes, batch, fanouts, model, dtype, &c.lay);
    if (rc != SDT_OK) return rc;
    rc = check_step_args("sdt_train_step", graph, X, ldx, labels, seeds, batch, model, loss_d);
    if (rc != SDT_OK) return rc;
    SDT_REQUIRE(ws && ws_bytes >= c.lay.total_bytes && aligned16(ws), SDT_ERR_WORKSPACE,
                "sdt_train_step: workspace of %llu bytes needed, %zu given", (unsigned long long)c.lay.total_bytes,
                ws_bytes);
    hipStream_t st = static_cast<hipStream_t>(stream);
    StepBuffers b;
    bind_buffers(c.lay, ws, ws_bytes, &b);
    c.slot = -1;
    if (timing) {
        if (timing->seen % timing->stride == 0 && timing->used < timing->max_steps) c.slot = timing->used++;
        ++timing->seen;
    }
    rc = step_sample(c, b, seeds, step, st);
    if (rc != SDT_OK) return rc;
    return step_compute(c, b, seeds, step, loss_d, st);
}

// Step workspaces the loop rotates through: the sampling phase may run this many steps ahead.
// The loop hands the two streams whole groups of steps: one pair of events per LOOP_GROUP steps instead
// of per step (every cross-stream wait costs a few microseconds of an ~100 us step).
static constexpr int LOOP_GROUP = 2;     // steps per hand-over
static constexpr int LOOP_SLOTS = 4;     // groups in flight: up to three being sampled, one being trained on
static constexpr int LOOP_MAX_AUX = LOOP_SLOTS - 1;
static constexpr int LOOP_BUFFERS = LOOP_GROUP * LOOP_SLOTS;

namespace sdt {
int32_t train_loop_buffers() { return LOOP_BUFFERS; }
}  // namespace sdt

namespace {
// Event sets of sdt_train_loop, kept for reuse per device (never destroyed: they live as long as the process).
struct LoopEvents {
    int dev = -1;
    hipEvent_t ready[LOOP_SLOTS] = {}, done[LOOP_SLOTS] = {}, fork = nullptr;
};
std::mutex loop_events_mu;
std::vector<LoopEvents*> loop_events_free;

LoopEvents* loop_events_acquire() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return nullptr;
    {
        std::lock_guard<std::mutex> lock(loop_events_mu);
        for (size_t k = 0; k < loop_events_free.size(); ++k)
            if (loop_events_free[k]->dev == dev) {
                LoopEvents* e = loop_events_free[k];
                loop_events_free.erase(loop_events_free.begin() + (long)k);
                return e;
            }
    }
    LoopEvents* e = new LoopEvents;
    e->dev = dev;
    bool ok = hipEventCreateWithFlags(&e->fork, hipEventDisableTiming) == hipSuccess;
    for (int k = 0; k < LOOP_SLOTS && ok; ++k)
        ok = hipEventCreateWithFlags(&e->ready[k], hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&e->done[k], hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        for (int k = 0; k < LOOP_SLOTS; ++k) {
            if (e->ready[k]) (void)hipEventDestroy(e->ready[k]);
            if (e->done[k]) (void)hipEventDestroy(e->done[k]);
        }
        if (e->fork) (void)hipEventDestroy(e->fork);
        delete e;
        return nullptr;
    }
    return e;
}
void loop_events_release(LoopEvents* e) {
    std::lock_guard<std::mutex> lock(loop_events_mu);
    loop_events_free.push_back(e);
}
}  // namespace

extern "C" size_t sdt_train_loop_workspace_bytes(int64_t n_nodes, int32_t batch, const int32_t* fanouts,
                                                 const sdt_model* model, int32_t dtype) {
    sdt_step_layout lay;
    if (sdt_train_step_layout(n_nodes, batch, fanouts, model, dtype, &lay) != SDT_OK) return 0;
    return LOOP_BUFFERS * align_up((size_t)lay.total_bytes, 256);
}

extern "C" int32_t sdt_train_loop(const sdt_csr* graph, const void* X, int64_t ldx, int32_t dtype, const int32_t* labels,
                                  const int32_t* seeds, int32_t batch, int32_t n_steps, const int32_t* fanouts,
                                  const sdt_model* model, uint64_t seed, uint32_t first_step, float lr, float* losses_d,
                                  sdt_timing* timing, void* ws, size_t ws_bytes, void* stream, void* const* aux_streams, int32_t n_aux) {
    SDT_REQUIRE(graph && graph->indptr, SDT_ERR_INVALID_ARG, "sdt_train_loop: null graph");
    SDT_REQUIRE(n_steps >= 0, SDT_ERR_INVALID_ARG, "sdt_train_loop: n_steps = %d", n_steps);
    StepCtx c{graph, X, ldx, dtype, labels, batch, fanouts, model, seed, lr, timing, {}};
    int32_t rc = sdt_train_step_layout(graph->n_nodes, batch, fanouts, model, dtype, &c.lay);
    if (rc != SDT_OK) return rc;
    rc = check_step_args("sdt_train_loop", graph, X, ldx, labels, seeds, batch, model, losses_d);
    if (rc != SDT_OK) return rc;
    const size_t one = align_up((size_t)c.lay.total_bytes, 256);
    SDT_REQUIRE(ws && ws_bytes >= LOOP_BUFFERS * one && aligned16(ws), SDT_ERR_WORKSPACE,
                "sdt_train_loop: workspace of %zu bytes needed, %zu given", LOOP_BUFFERS * one, ws_bytes);
    SDT_REQUIRE(n_aux >= 0 && n_aux <= LOOP_MAX_AUX && (n_aux == 0 || aux_streams), SDT_ERR_INVALID_ARG,
                "sdt_train_loop: n_aux = %d outside [0,%d] or null stream array", n_aux, LOOP_MAX_AUX);
    hipStream_t main_st = static_cast<hipStream_t>(stream);
    hipStream_t aux[LOOP_MAX_AUX] = {};
    for (int k = 0; k < n_aux; ++k) {
        aux[k] = static_cast<hipStream_t>(aux_streams[k]);
        SDT_REQUIRE(aux[k] != main_st, SDT_ERR_INVALID_ARG, "sdt_train_loop: auxiliary stream %d is the main stream", k);
    }
    // one or two steps are quicker in sequence than with helper threads and cross-stream waits set up
    // (measured: 152 against 247 us for one step, 297 against 351 us for two)
    const bool overlap = n_aux > 0 && n_steps > 2;
    StepBuffers buf[LOOP_BUFFERS];
    for (int k = 0; k < LOOP_BUFFERS; ++k) bind_buffers(c.lay, static_cast<char*>(ws) + k * one, one, &buf[k]);
    // the weight images of every step of this call live in the first workspace (see StepCtx::images)
    if (c.lay.wlow != 0 && model->kind == SDT_MODEL_SAGE_MEAN) c.images = static_cast<char*>(buf[0].at(c.lay.wlow));

    // ready[s]: phase 1 of every step of the group in slot s is complete; done[s]: their phase 2 is.
    // The events come from a pool and go back to it (creating and destroying nine of them costs a call
    // of a few dozen steps several percent); a set is used by one call at a time, and re-recording an
    // event does not disturb waits enqueued earlier, which refer to the record they were issued after.
    LoopEvents* ev = nullptr;
    hipEvent_t *ready = nullptr, *done = nullptr, fork = nullptr;
    auto cleanup = [&]() {
        if (ev) loop_events_release(ev);
        ev = nullptr;
    };
    if (overlap) {
        ev = loop_events_acquire();
        if (!ev) {
            set_error("sdt_train_loop: hipEventCreate failed");
            return SDT_ERR_HIP;
        }
        ready = ev->ready;
        done = ev->done;
        fork = ev->fork;
        // the auxiliary streams start after whatever the caller queued on the main stream
        (void)hipEventRecord(fork, main_st);
        for (int k = 0; k < n_aux; ++k) (void)hipStreamWaitEvent(aux[k], fork, 0);
    }
    rc = SDT_OK;
    // step i of this call is timed if it is a multiple of the stride among all steps the object has seen
    const int seen0 = timing ? timing->seen : 0, stride = timing ? timing->stride : 1;
    const int used0 = timing ? timing->used : 0;
    const int first_timed = (stride - seen0 % stride) % stride;   // first i with (seen0 + i) % stride == 0
    auto slot_of = [&](int i) {
        if (!timing || i < first_timed || (i - first_timed) % stride != 0) return -1;
        const int sl = used0 + (i - first_timed) / stride;
        return sl < timing->max_steps ? sl : -1;
    };
    // Groups of LOOP_GROUP steps, except the first, which is a single step: the model side can start as
    // soon as one step is sampled (a call pays the pipeline fill once; at a hundred steps per call it shows).
    // Step i still uses workspace i % LOOP_BUFFERS, and the steps of group g + LOOP_SLOTS use exactly the
    // workspaces of group g, so waiting for the slot's `done` event frees what the group needs.
    auto group_begin = [&](int g) { return g == 0 ? 0 : g * LOOP_GROUP - (LOOP_GROUP - 1); };
    auto group_end = [&](int g) { return group_begin(g + 1) < n_steps ? group_begin(g + 1) : n_steps; };
    const int n_groups = n_steps == 0 ? 0 : (n_steps - 1 + LOOP_GROUP - 1) / LOOP_GROUP + 1;
    if (!overlap) {
        for (int i = 0; i < n_steps && rc == SDT_OK; ++i) {
            c.slot = slot_of(i);
            c.images_current = i > 0;
            const StepBuffers& bi = buf[i % LOOP_BUFFERS];
            rc = step_sample(c, bi, seeds + (int64_t)i * batch, first_step + (uint32_t)i, main_st);
            if (rc == SDT_OK)
                rc = step_compute(c, bi, seeds + (int64_t)i * batch, first_step + (uint32_t)i, losses_d + i, main_st);
        }
    } else {
        // A step is about twenty launches and the host needs a few microseconds for each: one thread
        // cannot feed the GPU fast enough when the kernels are small.  So the sampling side is
        // enqueued by helper threads (one per auxiliary stream) and the model side by the calling thread.  A stream wait
        // refers to the event's latest record at the time of the CALL, so each side publishes
        // (group counters below) that it has recorded an event before the other side waits on it.
        std::atomic<int> ready_gen[LOOP_SLOTS], done_groups{0}, failed{0};
        for (int k = 0; k < LOOP_SLOTS; ++k) ready_gen[k].store(0);
        int dev = 0;
        (void)hipGetDevice(&dev);
        int32_t aux_rc[LOOP_MAX_AUX] = {};
        std::string aux_msg[LOOP_MAX_AUX];
        // one helper per auxiliary stream: helper a enqueues the groups g = a, a + n_aux, ... -- except group 0, the
        // call's first step, whose sampling the calling thread enqueues itself before it starts the helpers: the GPU
        // then works on it while the threads come up (their start is off the call's critical path)
        auto helper_fn = [&](int a) {
            (void)hipSetDevice(dev);
            StepCtx ca = c;
            hipStream_t aux_st = aux[a];
            for (int g = a == 0 ? n_aux : a; g < n_groups; g += n_aux) {
                const int s = g % LOOP_SLOTS;
                if (g >= LOOP_SLOTS) {
                    while (done_groups.load(std::memory_order_acquire) <= g - LOOP_SLOTS && !failed.load()) std::this_thread::yield();
                    if (failed.load()) return;
                    (void)hipStreamWaitEvent(aux_st, done[s], 0);   // the slot's buffers are free again
                }
                for (int i = group_begin(g); i < group_end(g); ++i) {
                    ca.slot = slot_of(i);
                    const int32_t r = step_sample(ca, buf[i % LOOP_BUFFERS], seeds + (int64_t)i * batch, first_step + (uint32_t)i,
                                                  aux_st);
                    if (r != SDT_OK) {
                        aux_rc[a] = r;
                        aux_msg[a] = sdt_last_error();
                        failed.store(1);
                        return;
                    }
                }
                (void)hipEventRecord(ready[s], aux_st);
                ready_gen[s].store(g + 1, std::memory_order_release);
            }
        };
        {   // group 0 (one step) on the first auxiliary stream
            c.slot = slot_of(0);
            rc = step_sample(c, buf[0], seeds, first_step, aux[0]);
            if (rc == SDT_OK) {
                (void)hipEventRecord(ready[0], aux[0]);
                ready_gen[0].store(1, std::memory_order_release);
            } else {
                failed.store(1);
            }
        }
        std::thread helpers[LOOP_MAX_AUX];
        int started = 0;
        if (rc == SDT_OK) try {
            for (int a = 0; a < n_aux; ++a) {
                helpers[a] = std::thread(helper_fn, a);
                ++started;
            }
        } catch (...) {   // no exception may cross the C boundary: stop the helpers already running and report
            failed.store(1);
            rc = SDT_ERR_HIP;
            set_error("sdt_train_loop: cannot start a helper thread");
        }
        for (int g = 0; g < n_groups && rc == SDT_OK; ++g) {
            const int s = g % LOOP_SLOTS;
            while (ready_gen[s].load(std::memory_order_acquire) != g + 1 && !failed.load()) std::this_thread::yield();
            if (failed.load()) break;
            (void)hipStreamWaitEvent(main_st, ready[s], 0);
            for (int i = group_begin(g); i < group_end(g) && rc == SDT_OK; ++i) {
                c.slot = slot_of(i);
                c.images_current = i > 0;
                rc = step_compute(c, buf[i % LOOP_BUFFERS], seeds + (int64_t)i * batch, first_step + (uint32_t)i, losses_d + i,
                                  main_st);
            }
            if (rc != SDT_OK) {
                failed.store(1);
                break;
            }
            (void)hipEventRecord(done[s], main_st);
            done_groups.store(g + 1, std::memory_order_release);
        }
        if (rc != SDT_OK) failed.store(1);
        for (int a = 0; a < started; ++a) helpers[a].join();
        for (int a = 0; a < started; ++a)
            if (rc == SDT_OK && aux_rc[a] != SDT_OK) {
                rc = aux_rc[a];
                set_error("%s", aux_msg[a].c_str());
            }
        if (rc != SDT_OK) {
            // sampling work of steps that no model phase waited for may still be queued on the auxiliary
            // streams: order the main stream after it, so that synchronising `stream` covers everything
            // this call enqueued on the failure path too
            for (int k = 0; k < n_aux; ++k) {
                (void)hipEventRecord(fork, aux[k]);
                (void)hipStreamWaitEvent(main_st, fork, 0);
            }
        }
    }
    if (timing) {
        const int timed = n_steps > first_timed ? (n_steps - first_timed + stride - 1) / stride : 0;
        timing->used = used0 + timed < timing->max_steps ? used0 + timed : timing->max_steps;
        timing->seen = seen0 + n_steps;
    }
    // every phase 1 was waited for by a phase 2 on the main stream, so synchronising the
    // main stream covers the auxiliary one; the events may be released now (pending work keeps
    // what it needs)
    cleanup();
    return rc;
}
