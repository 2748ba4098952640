/*
 * sdt.h -- C ABI of the MI355X (gfx950) per-worker GraphSAGE-mean training step.
 *
 * The operations are the ones a worker of the paper's training loop runs on
 * its own partition for every mini-batch (Sec. II-A "Distributed GNN
 * Training": graph sampling, neighbourhood aggregation, per-mini-batch
 * gradients; Sec. III-B: a partition keeps the full neighbour list of the
 * nodes it owns; Sec. III-E: sampler + graph store with feature data +
 * GraphSAGE model).  The paper fixes none of the details; the conventions are
 * stated per call below.
 *
 * General rules
 *  - Every function returns an sdt_status.  No exceptions, no aborts, nothing
 *    is printed.  sdt_last_error() gives a thread-local message for the last
 *    failing call on the calling thread.
 *  - Every pointer is a DEVICE pointer owned by the caller unless its comment
 *    says "host".  The library allocates and frees no device memory; scratch
 *    space is passed in as `ws`/`ws_bytes` (size from the matching
 *    *_workspace_bytes query, pure host arithmetic on the upper bounds;
 *    contents need no initialisation and are garbage afterwards).  Workspace
 *    and all row pointers must be 16-byte aligned.
 *  - What the library does hold between calls, all of it host-side or fixed at
 *    load time, none of it results: (1) sdt_train_loop keeps a process-wide pool
 *    of HIP events per device (nine per concurrent call, behind a mutex, never
 *    destroyed) and, for calls of more than two steps with auxiliary streams,
 *    starts one host thread per auxiliary stream and joins it before returning
 *    (the threads spin with yield on counters of the calling thread; if a thread
 *    cannot be started the call returns SDT_ERR_HIP); (2) two kernels that need
 *    more than 64 KB of LDS raise their limit once per process (atomic flags);
 *    (3) sdt_sage_linear_bwd_noalloc owns one device array per GPU and remembers
 *    its address per device; (4) the caller-owned sdt_timing objects.  Entry
 *    points may be called from several threads as long as calls that share a
 *    workspace, a timing object or the built-in scratch are ordered.
 *  - `stream` is a hipStream_t (NULL = default stream).  All work is enqueued
 *    asynchronously; no call synchronises with the host.  Outputs are valid
 *    once the stream has been synchronised.  Two calls that share a workspace
 *    must be ordered by the caller.
 *  - Sizes that depend on the data (frontier sizes, edge counts) stay on the
 *    device.  A row count is passed as a host upper bound `*_cap` (sizes the
 *    launch) plus an optional device scalar `*_d` holding the true count
 *    (NULL: the true count is the bound).
 *  - Leading dimensions (`ld*`) are in elements and may exceed the row width.
 *  - Node ids and block-local ids are int32; graph row offsets are int64.
 */
#ifndef SDT_H
#define SDT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sdt_status {
    SDT_OK = 0,
    SDT_ERR_INVALID_ARG = -1, /* null pointer, negative size, unknown dtype, fan-out out of range, overflow */
    SDT_ERR_WORKSPACE = -2,   /* ws too small or misaligned */
    SDT_ERR_HIP = -3          /* a HIP runtime call or launch failed */
} sdt_status;

typedef enum sdt_dtype {
    SDT_F32 = 0, /* IEEE binary32 */
    SDT_BF16 = 1 /* bfloat16 storage, fp32 accumulation */
} sdt_dtype;

#define SDT_MAX_LAYERS 8
#define SDT_MAX_FANOUT 64 /* one wavefront lane per sampled neighbour */

/* A partition's graph in CSR form.  Row v lists the neighbours of node v in
 * indices[indptr[v] .. indptr[v+1]).  Rows may contain self-loops and repeated
 * entries; a row must be shorter than 2^31. */
typedef struct sdt_csr {
    int64_t n_nodes;
    const int64_t *indptr;  /* [n_nodes + 1] */
    const int32_t *indices; /* [indptr[n_nodes]] */
} sdt_csr;

/* One sampled bipartite layer ("block").  Destination row i aggregates the
 * source rows cols[indptr[i] .. indptr[i+1]).  src_nodes lists the global id
 * of each source row; its first n_dst entries are the destination nodes in
 * their given order, the rest are the newly reached nodes in ascending id.
 * The transposed block (optional: pass both pointers or neither) lists for
 * source j the destination rows that use it, ascending.
 * counts = {n_dst, n_src, nnz, 0} on the device. */
typedef struct sdt_block {
    int32_t cap_dst;    /* host: upper bound on n_dst */
    int32_t cap_src;    /* host: capacity of src_nodes, >= min(cap_dst*(1+fanout), n_nodes) */
    int32_t cap_nnz;    /* host: capacity of cols / t_rows, >= cap_dst*fanout */
    int32_t reserved;
    int32_t *counts;    /* [4] */
    int32_t *indptr;    /* [cap_dst + 1] */
    int32_t *cols;      /* [cap_nnz] */
    int32_t *src_nodes; /* [cap_src] */
    int32_t *t_indptr;  /* [cap_src + 1] or NULL */
    int32_t *t_rows;    /* [cap_nnz] or NULL */
} sdt_block;

/* Model of L GraphSAGE-mean layers.  Layer l maps dims[l] -> dims[l+1]:
 * Z = H[:n_dst] W[l][0:in] + mean_neigh(H) W[l][in:2in] + b[l], ReLU on all
 * but the last layer.  W[l] is fp32 [2*dims[l], dims[l+1]] row-major (rows
 * 0..in-1 act on the node's own features), b[l] fp32 [dims[l+1]].
 * dW/db (same shapes, nullable per layer) receive the gradients. */
typedef struct sdt_model {
    int32_t n_layers;
    int32_t dims[SDT_MAX_LAYERS + 1];
    float *W[SDT_MAX_LAYERS];
    float *b[SDT_MAX_LAYERS];
    float *dW[SDT_MAX_LAYERS];
    float *db[SDT_MAX_LAYERS];
    /* SDT_MODEL_SAGE_MEAN (0, the default) or SDT_MODEL_GCN: layer l is
     * H' = act(Agcn(H) W[l] + b[l]) with ONE weight matrix W[l] fp32 [dims[l], dims[l+1]]
     * and the aggregation of sdt_gcn_aggregate_fwd; fp32 or bf16 storage, even dims[0..L-1] only. */
    int32_t kind;
    /* Optimiser of sdt_train_step: SDT_OPT_SGD (0, the default; w -= lr g) or SDT_OPT_ADAM:
     * m = beta1 m + (1-beta1) g, v = beta2 v + (1-beta2) g^2,
     * w -= lr (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps) with t = step + 1 (the step
     * argument of sdt_train_step counts updates from 0).  mW/vW (like W) and mb/vb (like b)
     * are the caller's fp32 moment buffers, zero before the first step.  (The paper does not
     * name its optimiser.) */
    int32_t optimizer;
    float beta1, beta2, eps;
    float gat_slope; /* SDT_MODEL_GAT: negative slope of the LeakyReLU on the attention scores (e.g. 0.2) */
    float *mW[SDT_MAX_LAYERS];
    float *vW[SDT_MAX_LAYERS];
    float *mb[SDT_MAX_LAYERS];
    float *vb[SDT_MAX_LAYERS];
    /* SDT_MODEL_GAT (Sec. III-E: GAT is one of the integrated models; one head): layer l is
     * H' = act(GATagg(H W[l]) + b[l]) with W[l] fp32 [dims[l], dims[l+1]] applied to EVERY
     * frontier row, the attention aggregation of sdt_gat_aggregate_fwd with
     * a_src = att[l][0:out], a_dst = att[l][out:2out], ReLU on all but the last layer.
     * att[l] fp32 [2*dims[l+1]] is trained like a bias: datt (nullable) receives its gradient,
     * matt/vatt are its Adam moments.  fp32 or bf16 storage (bf16: the gathered rows, z, the hidden
     * activations and the gradients w.r.t. them; scores, sums, logits and parameters stay fp32), even
     * dims[0..L-1] only. */
    float *att[SDT_MAX_LAYERS];
    float *datt[SDT_MAX_LAYERS];
    float *matt[SDT_MAX_LAYERS];
    float *vatt[SDT_MAX_LAYERS];
} sdt_model;
enum { SDT_MODEL_SAGE_MEAN = 0, SDT_MODEL_GCN = 1, SDT_MODEL_GAT = 2 };
enum { SDT_OPT_SGD = 0, SDT_OPT_ADAM = 1 };

/* Byte offsets, inside the sdt_train_step workspace, of everything the step
 * produces (so a caller can inspect it), plus the capacities they were sized
 * for.  Index l is the GNN layer (0 = input-most).  H[0] holds the gathered
 * input rows of layer 0's DESTINATION nodes only, [cap_dst[0], dims[0]] with row stride ld_in (the
 * other frontier rows are aggregated straight out of X and never copied);
 * H[l+1] the output of layer l (H[L] = logits,
 * always fp32); A[l] the mean-aggregated neighbours; dZ the loss gradient
 * w.r.t. the logits (fp32); dH[l] (l >= 1) the gradient w.r.t. H[l] with the
 * ReLU mask of layer l-1 already applied; dSelf/dAgg[l] (l >= 1) the input
 * gradients of layer l's projection; dW/db the weight gradients (fp32).
 * t_indptr/t_rows exist for l >= 1 only (layer 0 needs no input gradient). */
typedef struct sdt_step_layout {
    uint64_t total_bytes;
    uint64_t header; /* int32[64], reserved */
    uint64_t state;  /* frontier state of the step being built: node -> local-id map, two state bits per node, per-word ranks */
    int32_t n_layers;
    int32_t cap_dst[SDT_MAX_LAYERS];
    int32_t cap_src[SDT_MAX_LAYERS];
    int32_t cap_nnz[SDT_MAX_LAYERS];
    uint64_t counts[SDT_MAX_LAYERS];
    uint64_t indptr[SDT_MAX_LAYERS];
    uint64_t cols[SDT_MAX_LAYERS];
    uint64_t src_nodes[SDT_MAX_LAYERS];
    uint64_t t_indptr[SDT_MAX_LAYERS];
    uint64_t t_rows[SDT_MAX_LAYERS];
    uint64_t H[SDT_MAX_LAYERS + 1];
    uint64_t A[SDT_MAX_LAYERS];
    uint64_t dZ;
    uint64_t dH[SDT_MAX_LAYERS];
    uint64_t dSelf[SDT_MAX_LAYERS];
    uint64_t dAgg[SDT_MAX_LAYERS];
    uint64_t dW[SDT_MAX_LAYERS];
    uint64_t db[SDT_MAX_LAYERS];
    uint64_t row_loss; /* fp32 [B]: per-seed loss before the mean */
    uint64_t scratch;  /* internal */
    uint64_t wlow;     /* internal: bf16 images of the weights (bf16 workloads only) */
    uint64_t norm[SDT_MAX_LAYERS]; /* GCN only: fp32 c[cap_src] | s[cap_dst] | selfw[cap_dst], each 256-byte aligned */
    /* GAT only.  H[0] then holds EVERY frontier row of layer 0, [cap_src[0], dims[0]], H[l+1] is
     * act(attention output + b); z[l] = H[l] W[l] and dz[l] = d loss / d z[l] are
     * [cap_src[l], dims[l+1]] in the storage type; dH[l] (l >= 1) is d loss / d H[l] with the ReLU mask applied;
     * datt[l] fp32 [2*dims[l+1]]; t_indptr/t_rows exist for every layer; A, dSelf, dAgg are unused. */
    uint64_t z[SDT_MAX_LAYERS];
    uint64_t dz[SDT_MAX_LAYERS];
    uint64_t datt[SDT_MAX_LAYERS];
    uint64_t gatws[SDT_MAX_LAYERS]; /* internal */
    /* Row stride, in elements, of H[0] and A[0]: dims[0], or (GraphSAGE kind) dims[0] rounded up to
     * whole 128-byte lines when it is not one already, so that every input row starts on a line
     * and the projections read it in 16-byte vectors; the columns past dims[0] are kept zero.  Every other matrix is stored densely (stride = its width). */
    uint64_t ld_in;
} sdt_step_layout;

/* Library version as "major.minor.patch" (host string, static storage). */
const char *sdt_version(void);
/* Message of the last failing call on this thread (host string; "" if none). */
const char *sdt_last_error(void);
/* sizeof of a struct of this header as the library was compiled (a binding that mirrors the structs
 * checks itself against it): which = 0 sdt_csr, 1 sdt_block, 2 sdt_model, 3 sdt_step_layout,
 * 4 sdt_partition; 0 for any other value. */
size_t sdt_struct_bytes(int32_t which);

/* ---- sampling (Sec. II-A: mini-batch graph sampling; Sec. III-B: the full
 * neighbour list of every owned node is present in the partition) ----------
 * For each destination node v (distinct ids in [0, n_nodes)) with degree d:
 * take all d neighbours if d <= fanout, else `fanout` distinct CSR positions
 * chosen uniformly by a partial Fisher-Yates shuffle of the positions, step i
 * swapping position i with position i + floor(r_i (d - i) / 2^32), r_i the
 * Philox4x32-10 word (key = seed halves, counter = (i/4, v, layer, step),
 * word i%4).  Neighbours are emitted in ascending CSR position.  Then builds
 * the source frontier, local column ids, and (if requested) the transposed
 * block; writes out->counts.  0 <= fanout <= SDT_MAX_FANOUT.
 * Errors: INVALID_ARG for bad arguments or capacities below the bounds in
 * sdt_block; WORKSPACE if ws is too small. */
size_t sdt_sample_workspace_bytes(int64_t n_nodes, int32_t cap_dst, int32_t fanout);
int32_t sdt_sample_csr(const sdt_csr *graph /*host struct*/, const int32_t *dst_nodes, int32_t n_dst_cap,
                       const int32_t *n_dst_d, int32_t fanout, uint64_t seed, uint32_t step, uint32_t layer,
                       const sdt_block *out /*host struct*/, void *ws, size_t ws_bytes, void *stream);

/* ---- feature fetch (Sec. III-E: graph store holding the partition's node
 * features) --- out[j, 0:F] = X[idx[j], 0:F] for j < n, a bit copy.
 * idx values must lie inside X. */
int32_t sdt_gather_features(const void *X, int64_t ldx, int32_t F, int32_t dtype, const int32_t *idx,
                            int32_t n_cap, const int32_t *n_d, void *out, int64_t ldo, void *stream);

/* ---- neighbourhood aggregation (Sec. II-A, the operation every GNN layer is
 * built on), mean variant: A[i,:] = (1/m_i) sum_{e in row i} H[cols[e],:],
 * m_i = row length, zeros when m_i = 0; fp32 accumulation in edge order.
 * Uses blk->counts[0] rows. */
int32_t sdt_sage_aggregate_fwd(const sdt_block *blk /*host struct*/, const void *H, int64_t ldh, int32_t F,
                               int32_t dtype, void *A, int64_t lda, void *stream);
/* Gather and aggregate in one pass: A[i,:] = (1/m_i) sum_e X[src_nodes[cols[e]],:], reading the
 * partition's feature matrix X (leading dimension ldx) through the block's frontier, so that the
 * gathered copy of the frontier rows that are not destinations need not exist. */
int32_t sdt_sage_aggregate_gather_fwd(const sdt_block *blk /*host struct*/, const void *X, int64_t ldx, int32_t F,
                                      int32_t dtype, void *A, int64_t lda, void *stream);
/* Same over a whole graph with the identity frontier (layer-wise inference):
 * row v aggregates H[indices[e],:] over its CSR row. */
int32_t sdt_sage_aggregate_csr_fwd(const sdt_csr *graph /*host struct*/, const void *H, int64_t ldh, int32_t F,
                                   int32_t dtype, void *A, int64_t lda, void *stream);
/* Backward: dH[j,:] = [j < n_dst] dSelf[j,:] + sum over edges (i -> j) of
 * dAgg[i,:]/m_i, for j < n_src, gathered through the transposed block (no
 * atomics; deterministic).  dSelf may be NULL.  If relu_of != NULL the result
 * is zeroed wherever relu_of[j,f] <= 0 (the ReLU mask of the layer that
 * produced H; relu_of has the same dtype and leading dimension as dH).
 * dH is overwritten. */
int32_t sdt_sage_aggregate_bwd(const sdt_block *blk /*host struct*/, const void *dAgg, int64_t ldg,
                               const void *dSelf, int64_t lds, const void *relu_of, int32_t F, int32_t dtype,
                               void *dH, int64_t ldd, void *stream);

/* ---- GCN aggregation on a sampled block (Sec. III-E: GCN is one of the integrated models;
 * the paper does not say how it is normalised on sampled blocks) -------------------
 * With deg(v) the length of v's row in the partition graph and m_i the number of
 * sampled neighbours of destination i:
 *   c[j] = 1/sqrt(deg(j)+1) per source row, s[i] = (deg(i)/m_i)/sqrt(deg(i)+1) (0 if
 *   m_i = 0) and selfw[i] = 1/(deg(i)+1) per destination row           (sdt_gcn_norm)
 *   A[i,:] = s[i] * sum_{e in row i} c[col_e] * H[col_e,:] + selfw[i] * H[i,:]    (fwd)
 *   dH[j,:] = c[j] * sum_{(i -> j)} s[i] * dA[i,:] + [j < n_dst] selfw[j] * dA[j,:]  (bwd,
 *   through the transposed block; zeroed where relu_of <= 0 if relu_of != NULL).
 * With every neighbour sampled this is a row of D~^-1/2 (Adj + I) D~^-1/2 H.  H, A, dA, dH, relu_of in `dtype`
 * (fp32 or bf16, sums in fp32); c, s, selfw always fp32.
 * c has blk->cap_src floats, s and selfw blk->cap_dst.  through_src_nodes != 0: row r of
 * the block lives at H[src_nodes[r]] (H is the partition's feature matrix). */
int32_t sdt_gcn_norm(const sdt_csr *graph /*host struct*/, const sdt_block *blk /*host struct*/, float *c, float *s,
                     float *selfw, void *stream);
int32_t sdt_gcn_aggregate_fwd(const sdt_block *blk /*host struct*/, const void *H, int64_t ldh,
                              int32_t through_src_nodes, int32_t F, int32_t dtype, const float *c, const float *s,
                              const float *selfw, void *A, int64_t lda, void *stream);
int32_t sdt_gcn_aggregate_bwd(const sdt_block *blk /*host struct*/, const void *dA, int64_t lda, const void *relu_of,
                              int32_t F, int32_t dtype, const float *c, const float *s, const float *selfw, void *dH,
                              int64_t ldd, void *stream);

/* ---- GAT attention aggregation on a sampled block (Sec. III-E: GAT is one of the
 * integrated models; the variant is not described: one head, LeakyReLU slope argument,
 * and a self edge so that no softmax is empty) ----------------------------------------
 * z is the already projected feature matrix, [n_src, F] in `dtype` (row i < n_dst is
 * destination i itself); a_src, a_dst are fp32 [F].  out, g and dz are in `dtype` too (fp32 or
 * bf16: widened on load, rounded on store); scores, softmax and every sum are fp32.
 *   s_(i<-j) = LeakyReLU(a_dst . z_i + a_src . z_j) over row i's edges and j = i,
 *   alpha = softmax over that set, out[i,:] = sum alpha_(i<-j) z[j,:]          (forward)
 * The backward takes g = d loss / d out [n_dst, F] and writes dz [n_src, F] (overwritten),
 * da_src [F], da_dst [F]; it needs the transposed block and the SAME workspace, untouched,
 * that the matching forward call used (the forward leaves z a_src, z a_dst and each row's
 * log-sum-exp there).  Deterministic: no atomics, fixed summation orders. */
size_t sdt_gat_workspace_bytes(int32_t cap_src, int32_t cap_dst, int32_t F);
int32_t sdt_gat_aggregate_fwd(const sdt_block *blk /*host struct*/, const void *z, int64_t ldz, int32_t F, int32_t dtype,
                              const float *a_src, const float *a_dst, float slope, void *out, int64_t ldo, void *ws,
                              size_t ws_bytes, void *stream);
int32_t sdt_gat_aggregate_bwd(const sdt_block *blk /*host struct*/, const void *z, int64_t ldz, int32_t F, int32_t dtype,
                              const float *a_src, const float *a_dst, float slope, const void *g, int64_t ldg,
                              void *dz, int64_t lddz, float *da_src, float *da_dst, void *ws, size_t ws_bytes,
                              void *stream);

/* ---- GraphSAGE projection (Sec. III-E / IV-A: GraphSAGE is the model trained)
 * Y = act(Hself W[0:in,:] + A W[in:2in,:] + b), act = ReLU if relu else id.
 * Hself, A are `dtype`; W, b fp32 (rounded to bf16 as MFMA operands when
 * dtype is BF16); Y is `y_dtype`; accumulation fp32 on the matrix cores. */
int32_t sdt_sage_linear_fwd(const void *Hself, int64_t ldh, const void *A, int64_t lda, int32_t n_cap,
                            const int32_t *n_d, int32_t in, int32_t out, const float *W, const float *b,
                            int32_t relu, int32_t dtype, void *Y, int64_t ldy, int32_t y_dtype, void *stream);
/* One full-neighbour layer over a whole graph in ONE launch (Sec. IV-A: the evaluation pass runs
 * the trained model over every node's full neighbourhood):
 *   Y[v,:] = act(H[v,:] W[0:in,:] + mean_{u in row v} H[u,:] W[in:2in,:] + b),  zeros for the mean of an empty row.
 * The aggregated rows stay in LDS and never reach HBM; the result equals
 * sdt_sage_aggregate_csr_fwd followed by sdt_sage_linear_fwd bit for bit.  Supported shapes
 * (sdt_sage_layer_csr_fused_ok returns 1): fp32, in a multiple of 128, out a multiple of 4 up to 256;
 * H (leading dimension ldh, a multiple of 4) and W must be 16-byte aligned; other shapes return
 * SDT_ERR_INVALID_ARG and are served by the two calls.  b may be NULL.  No workspace. */
int32_t sdt_sage_layer_csr_fused_ok(int32_t in, int32_t out, int32_t dtype);
int32_t sdt_sage_layer_csr_fwd(const sdt_csr *graph /*host struct*/, const void *H, int64_t ldh, int32_t in, int32_t out,
                               const float *W, const float *b, int32_t relu, int32_t dtype, void *Y, int64_t ldy,
                               void *stream);
/* Backward.  dZ = dY masked by Y > 0 when relu (Y in `dtype`, may be NULL
 * otherwise); dW = [Hself|A]^T dZ (fp32 [2in,out]); db = column sums of dZ;
 * dSelf = dZ W[0:in]^T and dAgg = dZ W[in:2in]^T in `dtype` with leading
 * dimension ldi (pass both or neither).  dY is `dy_dtype`.  The reduction over
 * rows is split and summed in a fixed order (deterministic). */
size_t sdt_linear_bwd_workspace_bytes(int32_t n_cap, int32_t in, int32_t out);
int32_t sdt_sage_linear_bwd(const void *dY, int64_t lddy, int32_t dy_dtype, const void *Y, int64_t ldy,
                            int32_t relu, const void *Hself, int64_t ldh, const void *A, int64_t lda,
                            int32_t n_cap, const int32_t *n_d, int32_t in, int32_t out, const float *W,
                            int32_t dtype, float *dW, float *db, void *dSelf, void *dAgg, int64_t ldi,
                            void *ws, size_t ws_bytes, void *stream);
/* sdt_sage_linear_bwd for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * errors, without the workspace: the scratch (split partial products, bias partials, masked
 * copy of dY) is a device array of SDT_NOALLOC_SCRATCH_BYTES built into the library, one copy
 * per GPU, held until the process ends.  The call allocates and frees nothing and only launches
 * kernels on `stream`.  Shapes whose sdt_linear_bwd_workspace_bytes exceeds the built-in size
 * return SDT_ERR_WORKSPACE (use sdt_sage_linear_bwd then).  All calls on one GPU share that
 * GPU's array: calls that may overlap in time on one GPU (different streams, different threads)
 * race on it and must be ordered by the caller.  Nothing in the array has to start at zero: a
 * call writes every byte it later reads. */
#define SDT_NOALLOC_SCRATCH_BYTES (32u << 20)
int32_t sdt_sage_linear_bwd_noalloc(const void *dY, int64_t lddy, int32_t dy_dtype, const void *Y, int64_t ldy,
                                    int32_t relu, const void *Hself, int64_t ldh, const void *A, int64_t lda,
                                    int32_t n_cap, const int32_t *n_d, int32_t in, int32_t out, const float *W,
                                    int32_t dtype, float *dW, float *db, void *dSelf, void *dAgg, int64_t ldi,
                                    void *stream);

/* ---- the whole mini-batch step (Sec. II-A and III-D: local training on the
 * worker's partition between two model synchronisations) -------------------
 * blocks are sampled from the seeds outwards: layer L-1 uses fanouts[L-1] on
 * the seeds, layer l's sources are layer l-1's destinations; then gather,
 * forward, mean softmax cross-entropy over the B seeds against
 * labels[seeds[i]], backward, and W -= lr dW, b -= lr db (plain SGD on the
 * fp32 weights; lr = 0 leaves them bit-identical).  loss_d receives the loss.
 * X is [n_nodes, F = dims[0]] in `dtype` with leading dimension ldx.
 * Workspace: like the other calls' scratch, it needs no initialisation and carries
 * nothing from one step to the next -- every step rebuilds its frontier state from
 * nothing (two bits per node are cleared when it starts; the node -> local-id map is
 * read only where the same step wrote it) -- so the buffer may be used for anything
 * else between steps.  What a step leaves in it (blocks, activations, gradients; see
 * sdt_train_step_layout) stays readable until the next call that uses it.
 * sdt_train_step_layout fills `layout` (host) with the workspace size and
 * the offsets of every intermediate.
 * Without a timing object the call only launches kernels on `stream`: no
 * allocation, no copy from or to the host, no synchronisation and no memset
 * node, so it may be recorded into a HIP graph (stream capture) and replayed;
 * the graph then repeats the recorded (seeds pointer, seed, step, lr). */
/* Optional per-stage timing of sdt_train_step with HIP events recorded on the
 * step's own stream (for measurement; adds two event records per selected
 * stage).  A stage is (kind, layer); its bit in `stage_mask` is
 * kind * SDT_MAX_LAYERS + layer.  SAMPLE spans all kernels of one layer's
 * sampling; GATHER and LOSS use layer 0; LINEAR_BWD covers a layer's backward
 * products (the single reduction + SGD launch at the end of the step is not timed).  Each timed step consumes one
 * slot (at most max_steps; further steps are not timed).  sdt_timing_read
 * waits for the recorded events and writes one duration in milliseconds per
 * timed step to ms_out (host, capacity max_steps) and their number to *n_out.
 * All timing objects are host objects owned by the caller via create/destroy. */
typedef struct sdt_timing sdt_timing;
enum {
    SDT_STAGE_SAMPLE = 0,
    SDT_STAGE_GATHER = 1,
    SDT_STAGE_AGG_FWD = 2,
    SDT_STAGE_LINEAR_FWD = 3,
    SDT_STAGE_LOSS = 4,
    SDT_STAGE_LINEAR_BWD = 5,
    SDT_STAGE_AGG_BWD = 6,
    SDT_STAGE_HEAD = 7, /* the fused last-layer launch alone (it also lies inside LINEAR_BWD of that layer) */
    /* single launches inside the stages above, for kernel-level figures: */
    SDT_STAGE_SAMPLE_ROWS = 8,  /* the neighbour sampling kernel of a layer */
    SDT_STAGE_FRONT_SCAN = 9,   /* first pass of the frontier / row-offset scan */
    SDT_STAGE_FRONT_APPLY = 10, /* second pass: new frontier nodes, row offsets, node map */
    SDT_STAGE_RELABEL = 11,     /* global -> local column ids (+ column histogram) */
    SDT_STAGE_TRANSPOSE = 12,   /* the transposed block (one launch for small layers, five otherwise) */
    SDT_STAGE_UPDATE = 13,      /* layer 0 only: the step's single reduction + optimiser launch */
    SDT_STAGE_BWD_WEIGHT = 14,  /* the weight-gradient product of a layer's backward */
    SDT_STAGE_BWD_INPUT = 15    /* the input-gradient product of a layer's backward */
};
#define SDT_STAGE_MASK_WORDS 2 /* 16 stage kinds x SDT_MAX_LAYERS bits */
int32_t sdt_timing_create(int32_t max_steps, uint64_t stage_mask, sdt_timing **out /*host*/);
/* The same with the full mask: stage_mask is a host array of SDT_STAGE_MASK_WORDS words, bit
 * kind * SDT_MAX_LAYERS + layer counted across the words (sdt_timing_create reaches kinds 0..7 only). */
int32_t sdt_timing_create_wide(int32_t max_steps, const uint64_t *stage_mask /*host*/, sdt_timing **out /*host*/);
void sdt_timing_destroy(sdt_timing *t);
void sdt_timing_reset(sdt_timing *t);
/* Time only every stride-th step (default 1: all).  An event record costs the stream a few
 * microseconds, which matters when a whole step takes under a hundred.  Call before the first
 * timed step or right after a reset. */
int32_t sdt_timing_set_stride(sdt_timing *t, int32_t stride);
int32_t sdt_timing_read(sdt_timing *t, int32_t kind, int32_t layer, float *ms_out /*host*/, int32_t *n_out /*host*/);

int32_t sdt_train_step_layout(int64_t n_nodes, int32_t batch, const int32_t *fanouts /*host*/,
                              const sdt_model *model /*host struct; only n_layers, dims read*/, int32_t dtype,
                              sdt_step_layout *layout /*host*/);
int32_t sdt_train_step(const sdt_csr *graph /*host struct*/, const void *X, int64_t ldx, int32_t dtype,
                       const int32_t *labels, const int32_t *seeds, int32_t batch,
                       const int32_t *fanouts /*host*/, const sdt_model *model /*host struct*/, uint64_t seed,
                       uint32_t step, float lr, float *loss_d, sdt_timing *timing /*host, nullable*/, void *ws,
                       size_t ws_bytes, void *stream);

/* ---- a run of consecutive steps with sampling overlapped --------------------
 * Same result, bit for bit, as n_steps calls of sdt_train_step with step =
 * first_step + i, seeds + i*batch and loss_d = losses_d + i -- but the phase of
 * a step that needs no weights (sampling, frontier, gather) is enqueued on
 * the auxiliary streams (groups of consecutive steps alternate between them)
 * and runs a few steps ahead of the forward/backward phase on `stream`, rotating
 * through several step workspaces; streams hand over groups of steps, one pair of
 * events per group (Sec. II-A: the
 * mini-batch sub-graphs are independent of the model; Sec. III-D: a worker
 * trains many mini-batches between two synchronisations).  Ordering between
 * the streams uses HIP events taken from and returned to the library's pool.  When
 * the call returns, with or without an error, everything it enqueued on any stream is
 * ordered before later work on `stream`; synchronising `stream` is enough.
 * seeds is device int32[n_steps, batch]; losses_d device fp32[n_steps].  The
 * workspace (sdt_train_loop_workspace_bytes: a whole number of step workspaces,
 * each with sdt_train_step's layout rounded up to 256 bytes, back to back;
 * step i of a call uses workspace i modulo their number) needs no initialisation
 * either.  aux_streams is a HOST array of n_aux (0..3)
 * streams, all different from `stream`; n_aux = 0 gives the serial order.  The
 * sampling chain is a sequence of small latency-bound launches, so two auxiliary
 * streams sample twice as many steps per unit of time as one.
 * All streams must have the default priority. */
size_t sdt_train_loop_workspace_bytes(int64_t n_nodes, int32_t batch, const int32_t *fanouts /*host*/,
                                      const sdt_model *model /*host struct*/, int32_t dtype);
int32_t sdt_train_loop(const sdt_csr *graph /*host struct*/, const void *X, int64_t ldx, int32_t dtype,
                       const int32_t *labels, const int32_t *seeds, int32_t batch, int32_t n_steps,
                       const int32_t *fanouts /*host*/, const sdt_model *model /*host struct*/, uint64_t seed,
                       uint32_t first_step, float lr, float *losses_d, sdt_timing *timing /*host, nullable*/,
                       void *ws, size_t ws_bytes, void *stream, void *const *aux_streams /*host*/, int32_t n_aux);

/* ---- layer-wise full-neighbour inference (Sec. IV-A: trained models are scored on
 * nodes with all of their neighbours) ----------------------------------------------
 * For every layer l over ALL n_nodes rows: A = mean over the node's whole CSR row,
 * H' = act(H W[l][0:in] + A W[l][in:2in] + b[l]), ReLU on all but the last layer;
 * H_0 = X.  logits is device fp32 [n_nodes, dims[L]] with leading dimension ldl.
 * Hidden activations are kept in `dtype` (bf16: rounded as in the training step).
 * n_nodes must be below 2^31.  The workspace (size from the query; no state) holds
 * the aggregated rows and two hidden-activation buffers of n_nodes rows each.
 * GCN and GAT models run the layer of their training step with the whole graph as the
 * block (every node a destination, every neighbour kept: the GCN weights are those of
 * D~^-1/2 (Adj + I) D~^-1/2).  For these two kinds the graph must hold fewer than 2^31
 * edges, and the call reads the edge count back first: it synchronises `stream` once
 * (an error, not a fault, if there are more). */
size_t sdt_infer_layerwise_workspace_bytes(int64_t n_nodes, const sdt_model *model /*host struct*/, int32_t dtype);
int32_t sdt_infer_layerwise(const sdt_csr *graph /*host struct*/, const void *X, int64_t ldx, int32_t dtype,
                            const sdt_model *model /*host struct*/, float *logits, int64_t ldl, void *ws,
                            size_t ws_bytes, void *stream);

/* ---- model synchronisation by weighted averaging (Sec. III-D) --------------------
 * out[e] = sum_i alpha[i] * params[i][e] for e < n_elems, accumulated in fp32 in the
 * order i = 0, 1, ... (deterministic).  In the paper alpha_i is worker i's share of
 * the training nodes; the caller passes the weights.  params is a HOST array of
 * n_models (1..64) device pointers, alpha a HOST array; out may be one of params[i]. */
int32_t sdt_model_average(const float *const *params /*host array of device pointers*/,
                          const float *alpha /*host*/, int32_t n_models, int64_t n_elems, float *out,
                          void *stream);

/* ---- one synchronisation round on a GPU that holds several partitions (Sec. III-C:
 * with more partitions than GPUs a GPU trains the local models of its partitions one
 * after the other; Sec. III-D: all local models are then averaged in proportion to
 * their numbers of training nodes) ---------------------------------------------------
 * For each partition j: local[j] <- global (weights and biases, and the attention
 * vectors of a GAT model, copied), then
 * sdt_train_loop on partition j with local[j] for its n_steps mini-batches (step
 * counter first_step + i); finally global <- sum_j alpha_j local[j] with
 * alpha_j = n_train_j / sum n_train.  losses_d receives sum_j n_steps_j losses,
 * partition after partition.  `locals` are caller-allocated models of the same
 * kind and shape as `global_model` (any of the three kinds).  ws must hold sdt_train_loop's workspace for the largest
 * partition (sdt_train_round_workspace_bytes). */
typedef struct sdt_partition {
    sdt_csr graph;
    const void *X;         /* [graph.n_nodes, dims[0]] in the round's dtype */
    int64_t ldx;
    const int32_t *labels; /* [graph.n_nodes] */
    const int32_t *seeds;  /* device int32 [n_steps, batch] */
    int32_t n_steps;
    int32_t reserved;
    int64_t n_train;       /* number of training nodes: the averaging weight */
} sdt_partition;
size_t sdt_train_round_workspace_bytes(const sdt_partition *parts /*host*/, int32_t n_parts, int32_t batch,
                                       const int32_t *fanouts /*host*/, const sdt_model *model /*host*/,
                                       int32_t dtype);
int32_t sdt_train_round(const sdt_partition *parts /*host*/, int32_t n_parts, int32_t dtype, int32_t batch,
                        const int32_t *fanouts /*host*/, const sdt_model *global_model /*host struct*/,
                        const sdt_model *locals /*host array of n_parts structs*/, uint64_t seed,
                        uint32_t first_step, float lr, float *losses_d, void *ws, size_t ws_bytes, void *stream,
                        void *const *aux_streams /*host*/, int32_t n_aux);

#ifdef __cplusplus
}
#endif
#endif /* SDT_H */
