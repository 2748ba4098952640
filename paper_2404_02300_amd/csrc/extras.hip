// Around the mini-batch step: layer-wise full-neighbour inference over a whole partition,
// weighted model averaging, and one synchronisation round over several partitions held by
// one GPU.  All three are chains of the step's own kernels plus one small averaging kernel.
#include "common.h"

namespace sdt {
namespace {

constexpr int MAX_MODELS = 64;
struct AvgArgs {
    const float* p[MAX_MODELS];
    float alpha[MAX_MODELS];
    int32_t n;
};

__global__ __launch_bounds__(256) void k_model_average(AvgArgs a, int64_t n_elems, float* __restrict__ out) {
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n_elems; e += (int64_t)gridDim.x * blockDim.x) {
        float acc = 0.f;
        for (int i = 0; i < a.n; ++i) acc += a.alpha[i] * a.p[i][e];
        out[e] = acc;
    }
}

// The whole graph as the block of a layer (GCN and GAT inference): every node a destination and a source,
// its CSR row the edges.  The kernels of those kinds take 32-bit row offsets and the counts on the device;
// for GCN the normalisation of a block in which every neighbour is kept (c = s = 1/sqrt(deg + 1), s = 0 for a
// node without neighbours, selfw = 1/(deg + 1)).  c, s, selfw may be null.
__global__ __launch_bounds__(256) void k_whole_graph_block(const int64_t* __restrict__ indptr, int n, int32_t* __restrict__ indptr32,
                                                           int32_t* __restrict__ counts, float* __restrict__ c,
                                                           float* __restrict__ s, float* __restrict__ selfw) {
    for (int v = blockIdx.x * 256 + threadIdx.x; v <= n; v += gridDim.x * 256) {
        const int64_t e0 = indptr[v];
        indptr32[v] = (int32_t)e0;
        if (v < n && c) {
            const float deg = (float)(indptr[v + 1] - e0);
            const float r = 1.0f / sqrtf(deg + 1.0f);
            c[v] = r;
            s[v] = deg > 0.f ? r : 0.f;
            selfw[v] = 1.0f / (deg + 1.0f);
        }
        if (v == n) {
            counts[0] = n;
            counts[1] = n;
            counts[2] = (int32_t)e0;
            counts[3] = 0;
        }
    }
}

struct InferWs {
    size_t a_off, h_off[2], w_off, total;
    size_t ip_off, cnt_off, norm_off[3], gat_off, gat_len;   // GCN / GAT kinds only
};
InferWs infer_ws(int64_t n_nodes, const sdt_model* m, int32_t dtype) {
    const size_t es = dtype_size(dtype);
    int32_t max_in = 0, max_hidden = 0, max_out = 0;
    size_t wb = 0, gat_len = 0;
    for (int l = 0; l < m->n_layers; ++l) {
        if (m->dims[l] > max_in) max_in = m->dims[l];
        if (l + 1 < m->n_layers && m->dims[l + 1] > max_hidden) max_hidden = m->dims[l + 1];
        if (m->dims[l + 1] > max_out) max_out = m->dims[l + 1];
        if (dtype == SDT_BF16 && m->kind == SDT_MODEL_SAGE_MEAN) wb += bf16_weights_bytes(m->dims[l], m->dims[l + 1]);
        if (m->kind == SDT_MODEL_GAT) {
            const size_t g = sdt_gat_workspace_bytes((int32_t)n_nodes, (int32_t)n_nodes, m->dims[l + 1]);
            if (g > gat_len) gat_len = g;
        }
    }
    InferWs w{};
    Arena a(nullptr);
    // the operand of the projection: the aggregated rows (GraphSAGE, GCN), or its result, the projected rows (GAT)
    w.a_off = a.take_off((size_t)n_nodes * (m->kind == SDT_MODEL_GAT ? max_out : max_in) * es);
    w.h_off[0] = a.take_off((size_t)n_nodes * (max_hidden > 0 ? max_hidden : 1) * es);
    w.h_off[1] = a.take_off((size_t)n_nodes * (max_hidden > 0 ? max_hidden : 1) * es);
    w.w_off = a.take_off(wb);
    if (m->kind != SDT_MODEL_SAGE_MEAN) {
        w.ip_off = a.take_off(((size_t)n_nodes + 1) * sizeof(int32_t));
        w.cnt_off = a.take_off(4 * sizeof(int32_t));
        if (m->kind == SDT_MODEL_GCN)
            for (int k = 0; k < 3; ++k) w.norm_off[k] = a.take_off((size_t)n_nodes * sizeof(float));
        w.gat_len = gat_len;
        w.gat_off = a.take_off(gat_len);
    }
    w.total = a.off;
    return w;
}

// rows of layer l's weight matrix: [self | neighbour] halves for GraphSAGE, one block for GCN and GAT
inline int64_t weight_rows(const sdt_model* m, int l) { return (m->kind == SDT_MODEL_SAGE_MEAN ? 2 : 1) * (int64_t)m->dims[l]; }

int32_t check_model_ptrs(const sdt_model* m, const char* who) {
    SDT_REQUIRE(m && m->n_layers >= 1 && m->n_layers <= SDT_MAX_LAYERS, SDT_ERR_INVALID_ARG, "%s: bad model", who);
    for (int l = 0; l < m->n_layers; ++l)
        SDT_REQUIRE(m->dims[l] > 0 && m->dims[l + 1] > 0 && m->W[l] && m->b[l] && (m->kind != SDT_MODEL_GAT || m->att[l]),
                    SDT_ERR_INVALID_ARG, "%s: layer %d has a null tensor or an empty dimension", who, l);
    return SDT_OK;
}

// Layer-wise inference of the GCN and GAT kinds: the layer of their training step with the whole graph as its block.
int32_t infer_single_matrix_kinds(const sdt_csr* graph, const void* X, int64_t ldx, int32_t dtype, const sdt_model* model,
                                  float* logits, int64_t ldl, char* base, const InferWs& w, hipStream_t st) {
    const int32_t N = (int32_t)graph->n_nodes;
    const int L = model->n_layers;
    const int32_t* d = model->dims;
    const size_t es = dtype_size(dtype);
    SDT_REQUIRE(graph->indices, SDT_ERR_INVALID_ARG, "sdt_infer_layerwise: null graph indices");
    // the blocks of these kinds count edges in 32 bits: read the edge count once (this synchronises the stream)
    int64_t nnz = 0;
    if (hipMemcpyAsync(&nnz, graph->indptr + N, sizeof(nnz), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        set_error("sdt_infer_layerwise: reading the edge count failed");
        return SDT_ERR_HIP;
    }
    SDT_REQUIRE(nnz >= 0 && nnz < 0x7FFFFFFF, SDT_ERR_INVALID_ARG,
                "sdt_infer_layerwise: %lld edges; the GCN and GAT kinds need fewer than 2^31", (long long)nnz);
    sdt_block blk{};
    blk.cap_dst = blk.cap_src = N;
    blk.cap_nnz = (int32_t)nnz;
    blk.counts = reinterpret_cast<int32_t*>(base + w.cnt_off);
    blk.indptr = reinterpret_cast<int32_t*>(base + w.ip_off);
    blk.cols = const_cast<int32_t*>(graph->indices);   // read only
    const bool gcn = model->kind == SDT_MODEL_GCN;
    float* c = gcn ? reinterpret_cast<float*>(base + w.norm_off[0]) : nullptr;
    float* s = gcn ? reinterpret_cast<float*>(base + w.norm_off[1]) : nullptr;
    float* selfw = gcn ? reinterpret_cast<float*>(base + w.norm_off[2]) : nullptr;
    const int64_t blocks = ((int64_t)N + 256) / 256;
    hipLaunchKernelGGL(k_whole_graph_block, dim3(blocks > 2048 ? 2048 : (int)blocks), dim3(256), 0, st, graph->indptr, N, blk.indptr,
                       blk.counts, c, s, selfw);
    SDT_CHECK_LAUNCH("whole-graph block");
    const char* H = static_cast<const char*>(X);
    int64_t ldh = ldx;
    int32_t rc;
    for (int l = 0; l < L; ++l) {
        const bool last = l == L - 1;
        const int F = d[l + 1];
        void* Y = last ? static_cast<void*>(logits) : static_cast<void*>(base + w.h_off[l & 1]);
        const int64_t ldy = last ? ldl : F;
        const int32_t y_dtype = last ? SDT_F32 : dtype;
        char* T = base + w.a_off;
        if (gcn) {
            rc = gcn_aggregate_fwd(&blk, H, ldh, false, d[l], dtype, c, s, selfw, T, d[l], st);
            if (rc != SDT_OK) return rc;
            rc = linear_fwd(T, d[l], T + (size_t)(d[l] / 2) * es, d[l], N, nullptr, d[l] / 2, F, model->W[l], model->b[l],
                            last ? 0 : 1, dtype, Y, ldy, y_dtype, false, st);
        } else {
            rc = linear_fwd(H, ldh, H + (size_t)(d[l] / 2) * es, ldh, N, nullptr, d[l] / 2, F, model->W[l], nullptr, 0, dtype, T, F,
                            dtype, false, st);
            if (rc != SDT_OK) return rc;
            rc = gat_forward(&blk, T, F, F, dtype, model->att[l], model->att[l] + F, model->gat_slope, model->b[l], last ? 0 : 1, Y,
                             ldy, y_dtype, base + w.gat_off, w.gat_len, st);
        }
        if (rc != SDT_OK) return rc;
        H = static_cast<const char*>(Y);
        ldh = ldy;
    }
    return SDT_OK;
}

}  // namespace
}  // namespace sdt

using namespace sdt;

extern "C" size_t sdt_infer_layerwise_workspace_bytes(int64_t n_nodes, const sdt_model* model, int32_t dtype) {
    if (!model || n_nodes < 0 || n_nodes >= 0x7FFFFFFF || !dtype_ok(dtype) || model->n_layers < 1 ||
        model->n_layers > SDT_MAX_LAYERS)
        return 0;
    return infer_ws(n_nodes, model, dtype).total;
}

extern "C" int32_t sdt_infer_layerwise(const sdt_csr* graph, const void* X, int64_t ldx, int32_t dtype,
                                       const sdt_model* model, float* logits, int64_t ldl, void* ws, size_t ws_bytes,
                                       void* stream) {
    int32_t rc = check_model_ptrs(model, "sdt_infer_layerwise");
    if (rc != SDT_OK) return rc;
    SDT_REQUIRE(graph && graph->indptr && dtype_ok(dtype), SDT_ERR_INVALID_ARG, "sdt_infer_layerwise: null graph or dtype");
    const int32_t kind = model->kind;
    SDT_REQUIRE(kind == SDT_MODEL_SAGE_MEAN || kind == SDT_MODEL_GCN || kind == SDT_MODEL_GAT, SDT_ERR_INVALID_ARG,
                "sdt_infer_layerwise: unknown model kind %d", kind);
    SDT_REQUIRE(kind != SDT_MODEL_GAT || (model->gat_slope >= 0.f && model->gat_slope <= 1.f), SDT_ERR_INVALID_ARG,
                "sdt_infer_layerwise: gat_slope %g outside [0,1]", (double)model->gat_slope);
    if (kind != SDT_MODEL_SAGE_MEAN)
        for (int l = 0; l < model->n_layers; ++l)
            SDT_REQUIRE(model->dims[l] % 2 == 0, SDT_ERR_INVALID_ARG,
                        "sdt_infer_layerwise: GCN and GAT need even layer input widths (dims[%d] = %d)", l, model->dims[l]);
    const int64_t N = graph->n_nodes;
    SDT_REQUIRE(N >= 0 && N < 0x7FFFFFFF, SDT_ERR_INVALID_ARG, "sdt_infer_layerwise: n_nodes %lld out of range",
                (long long)N);
    if (N == 0) return SDT_OK;
    const int L = model->n_layers;
    const int32_t* d = model->dims;
    SDT_REQUIRE(X && logits && ldx >= d[0] && ldl >= d[L], SDT_ERR_INVALID_ARG,
                "sdt_infer_layerwise: null tensor or leading dimension too small");
    const InferWs w = infer_ws(N, model, dtype);
    SDT_REQUIRE(ws && ws_bytes >= w.total && aligned16(ws), SDT_ERR_WORKSPACE,
                "sdt_infer_layerwise: workspace of %zu bytes needed, %zu given", w.total, ws_bytes);
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(ws);
    if (kind != SDT_MODEL_SAGE_MEAN) return infer_single_matrix_kinds(graph, X, ldx, dtype, model, logits, ldl, base, w, st);
    const char* wt[SDT_MAX_LAYERS] = {};
    if (dtype == SDT_BF16) {
        rc = convert_weights_bf16(model, base + w.w_off, st);
        if (rc != SDT_OK) return rc;
        const char* p = base + w.w_off;
        for (int l = 0; l < L; ++l) {
            wt[l] = p;
            p += bf16_weights_bytes(d[l], d[l + 1]);
        }
    }
    const void* H = X;
    int64_t ldh = ldx;
    for (int l = 0; l < L; ++l) {
        void* A = base + w.a_off;
        rc = sdt_sage_aggregate_csr_fwd(graph, H, ldh, d[l], dtype, A, d[l], stream);
        if (rc != SDT_OK) return rc;
        const bool last = l == L - 1;
        void* Y = last ? static_cast<void*>(logits) : static_cast<void*>(base + w.h_off[l & 1]);
        const int64_t ldy = last ? ldl : d[l + 1];
        if (dtype == SDT_BF16 && bf16_mfma_fwd_ok(H, ldh, A, d[l], d[l]))
            rc = linear_fwd_bf16(H, ldh, A, d[l], (int32_t)N, nullptr, d[l], d[l + 1], wt[l], model->b[l], last ? 0 : 1, Y, ldy,
                                 last ? SDT_F32 : dtype, st);
        else
            rc = sdt_sage_linear_fwd(H, ldh, A, d[l], (int32_t)N, nullptr, d[l], d[l + 1], model->W[l], model->b[l],
                                     last ? 0 : 1, dtype, Y, ldy, last ? SDT_F32 : dtype, stream);
        if (rc != SDT_OK) return rc;
        H = Y;
        ldh = ldy;
    }
    return SDT_OK;
}

extern "C" int32_t sdt_model_average(const float* const* params, const float* alpha, int32_t n_models, int64_t n_elems,
                                     float* out, void* stream) {
    SDT_REQUIRE(params && alpha && out && n_models >= 1 && n_models <= MAX_MODELS && n_elems >= 0, SDT_ERR_INVALID_ARG,
                "sdt_model_average: null argument or n_models outside [1,%d]", MAX_MODELS);
    if (n_elems == 0) return SDT_OK;
    AvgArgs a{};
    a.n = n_models;
    for (int i = 0; i < n_models; ++i) {
        SDT_REQUIRE(params[i], SDT_ERR_INVALID_ARG, "sdt_model_average: params[%d] is null", i);
        a.p[i] = params[i];
        a.alpha[i] = alpha[i];
    }
    const int blocks = (int)((n_elems + 255) / 256 < 4096 ? (n_elems + 255) / 256 : 4096);
    hipLaunchKernelGGL(k_model_average, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), a, n_elems, out);
    SDT_CHECK_LAUNCH("model_average");
    return SDT_OK;
}

extern "C" size_t sdt_train_round_workspace_bytes(const sdt_partition* parts, int32_t n_parts, int32_t batch,
                                                  const int32_t* fanouts, const sdt_model* model, int32_t dtype) {
    if (!parts || n_parts < 1) return 0;
    size_t m = 0;
    for (int j = 0; j < n_parts; ++j) {
        const size_t b = sdt_train_loop_workspace_bytes(parts[j].graph.n_nodes, batch, fanouts, model, dtype);
        if (b == 0) return 0;
        if (b > m) m = b;
    }
    return m;
}

extern "C" int32_t sdt_train_round(const sdt_partition* parts, int32_t n_parts, int32_t dtype, int32_t batch,
                                   const int32_t* fanouts, const sdt_model* global_model, const sdt_model* locals,
                                   uint64_t seed, uint32_t first_step, float lr, float* losses_d, void* ws,
                                   size_t ws_bytes, void* stream, void* const* aux_streams, int32_t n_aux) {
    int32_t rc = check_model_ptrs(global_model, "sdt_train_round");
    if (rc != SDT_OK) return rc;
    SDT_REQUIRE(parts && locals && n_parts >= 1 && n_parts <= MAX_MODELS, SDT_ERR_INVALID_ARG,
                "sdt_train_round: n_parts outside [1,%d] or null argument", MAX_MODELS);
    const int L = global_model->n_layers;
    double total = 0;
    for (int j = 0; j < n_parts; ++j) {
        rc = check_model_ptrs(&locals[j], "sdt_train_round (local model)");
        if (rc != SDT_OK) return rc;
        SDT_REQUIRE(locals[j].n_layers == L && locals[j].kind == global_model->kind, SDT_ERR_INVALID_ARG,
                    "sdt_train_round: local model %d has another depth or kind", j);
        for (int l = 0; l <= L; ++l)
            SDT_REQUIRE(locals[j].dims[l] == global_model->dims[l], SDT_ERR_INVALID_ARG,
                        "sdt_train_round: local model %d has another shape", j);
        SDT_REQUIRE(parts[j].n_train >= 0 && parts[j].n_steps >= 0, SDT_ERR_INVALID_ARG,
                    "sdt_train_round: partition %d has a negative count", j);
        total += (double)parts[j].n_train;
    }
    SDT_REQUIRE(total > 0, SDT_ERR_INVALID_ARG, "sdt_train_round: no training nodes at all");
    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t done = 0;
    for (int j = 0; j < n_parts; ++j) {
        // every local model starts the round from the synchronised weights
        for (int l = 0; l < L; ++l) {
            const size_t wb = (size_t)weight_rows(global_model, l) * global_model->dims[l + 1] * sizeof(float);
            const size_t bb = (size_t)global_model->dims[l + 1] * sizeof(float);
            const bool gat = global_model->kind == SDT_MODEL_GAT;   // ... and its attention vectors [a_src | a_dst]
            if (hipMemcpyAsync(locals[j].W[l], global_model->W[l], wb, hipMemcpyDeviceToDevice, st) != hipSuccess ||
                hipMemcpyAsync(locals[j].b[l], global_model->b[l], bb, hipMemcpyDeviceToDevice, st) != hipSuccess ||
                (gat && hipMemcpyAsync(locals[j].att[l], global_model->att[l], 2 * bb, hipMemcpyDeviceToDevice, st) != hipSuccess)) {
                set_error("sdt_train_round: copying the synchronised weights failed");
                return SDT_ERR_HIP;
            }
        }
        if (parts[j].n_steps > 0) {
            // (a step workspace carries nothing from one step to the next, so partitions with different
            // layouts may follow each other in the same buffer)
            rc = sdt_train_loop(&parts[j].graph, parts[j].X, parts[j].ldx, dtype, parts[j].labels, parts[j].seeds, batch,
                                parts[j].n_steps, fanouts, &locals[j], seed, first_step, lr, losses_d + done, nullptr, ws,
                                ws_bytes, stream, aux_streams, n_aux);
            if (rc != SDT_OK) return rc;
        }
        done += parts[j].n_steps;
    }
    // w = sum_j alpha_j w_j, tensor by tensor
    float alpha[MAX_MODELS];
    for (int j = 0; j < n_parts; ++j) alpha[j] = (float)((double)parts[j].n_train / total);
    const float* src[MAX_MODELS];
    for (int l = 0; l < L; ++l) {
        for (int j = 0; j < n_parts; ++j) src[j] = locals[j].W[l];
        rc = sdt_model_average(src, alpha, n_parts, weight_rows(global_model, l) * global_model->dims[l + 1],
                               global_model->W[l], stream);
        if (rc != SDT_OK) return rc;
        for (int j = 0; j < n_parts; ++j) src[j] = locals[j].b[l];
        rc = sdt_model_average(src, alpha, n_parts, global_model->dims[l + 1], global_model->b[l], stream);
        if (rc != SDT_OK) return rc;
        if (global_model->kind == SDT_MODEL_GAT) {
            for (int j = 0; j < n_parts; ++j) src[j] = locals[j].att[l];
            rc = sdt_model_average(src, alpha, n_parts, 2 * (int64_t)global_model->dims[l + 1], global_model->att[l], stream);
            if (rc != SDT_OK) return rc;
        }
    }
    return SDT_OK;
}
