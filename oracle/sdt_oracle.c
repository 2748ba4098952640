/*
 * CPU oracle for the per-worker mini-batch GraphSAGE-mean training step.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT: plain, slow, single-threaded C with fp64
 * arithmetic.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code with the HIP library.
 *
 * What it follows.  The paper (Sec. II-A "Distributed GNN Training" and
 * Sec. III-E "Implementation") says only that a worker samples mini-batch
 * sub-graphs from its partition, fetches their features, runs neighbourhood
 * aggregation in a GraphSAGE model and computes gradients per mini-batch; it
 * fixes no sampler, RNG, activation or optimiser.  Every function below is
 * therefore the textbook definition written out (mean aggregation, affine
 * projection, softmax cross-entropy, their exact derivatives, plain SGD),
 * and the sampler is a stated rule: partial Fisher-Yates over the CSR
 * positions of a row, driven by the published Philox4x32-10 generator with a
 * stated counter layout.  Those conventions are pinned only by agreement
 * between this file and the HIP path ("parity unpinned" as conventions); the
 * functions themselves are pinned by the CPU tests (known-answer vectors,
 * invariants, brute force, hand graphs, finite differences).
 *
 * Build: gcc -O2 -shared -fPIC sdt_oracle.c -o libsdt_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
 * as easy as 1, 2, 3", SC'11).  One round maps
 *   (c0,c1,c2,c3) -> (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0))
 * and then bumps the key by the Weyl constants.                        */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = M0 * c0;
        uint64_t prod1 = M1 * c2;
        uint32_t y0 = (uint32_t)(prod1 >> 32) ^ c1 ^ k0;
        uint32_t y1 = (uint32_t)prod1;
        uint32_t y2 = (uint32_t)(prod0 >> 32) ^ c3 ^ k1;
        uint32_t y3 = (uint32_t)prod0;
        c0 = y0; c1 = y1; c2 = y2; c3 = y3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Random word for (seed, step, layer, node, slot) in the neighbour-sampling
 * domain (domain 0): key = the two halves of seed, counter =
 * (slot/4, node, layer | domain<<16, step), word slot%4 of the block.     */
static uint32_t sample_word(uint64_t seed, uint32_t step, uint32_t layer, uint32_t node, uint32_t slot)
{
    uint32_t ctr[4] = { slot >> 2, node, layer | (0u << 16), step };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return out[slot & 3u];
}

/* ------------------------------------------------------------------ */
/* Sampling rule for one destination row of degree d with fan-out k.
 * d <= k: every position 0..d-1.  Otherwise k steps of Fisher-Yates on the
 * virtual array a[t] = t: at step i draw j uniformly in [i, d) as
 * i + floor(r_i * (d-i) / 2^32), output a[j], then a[j] <- a[i].
 * The chosen positions are returned in ascending order.  Returns min(d,k). */
int32_t orc_sample_positions(int64_t d, int32_t k, uint64_t seed, uint32_t step, uint32_t layer,
                             uint32_t node, int64_t *pos)
{
    if (k <= 0 || d <= 0) return 0;
    if (d <= k) {
        for (int64_t t = 0; t < d; ++t) pos[t] = t;
        return (int32_t)d;
    }
    /* entries of a[] that differ from the identity */
    int64_t *where = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    int64_t *value = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    int n_changed = 0;
    for (int32_t i = 0; i < k; ++i) {
        uint32_t r = sample_word(seed, step, layer, node, (uint32_t)i);
        int64_t j = i + (int64_t)(((uint64_t)r * (uint64_t)(d - i)) >> 32);
        int64_t a_j = j, a_i = i;
        int slot_j = -1;
        for (int t = 0; t < n_changed; ++t) {
            if (where[t] == j) { a_j = value[t]; slot_j = t; }
            if (where[t] == i) a_i = value[t];
        }
        pos[i] = a_j;
        if (slot_j < 0) { slot_j = n_changed++; where[slot_j] = j; }
        value[slot_j] = a_i;
    }
    free(where);
    free(value);
    for (int32_t i = 1; i < k; ++i) {           /* insertion sort, ascending */
        int64_t x = pos[i];
        int32_t t = i - 1;
        while (t >= 0 && pos[t] > x) { pos[t + 1] = pos[t]; --t; }
        pos[t + 1] = x;
    }
    return k;
}

/* Sample every destination row.  b_indptr[n_dst+1] receives the row offsets,
 * e_glob (capacity n_dst*fanout) the sampled neighbours' global ids in row
 * order.  Returns the number of sampled edges.                            */
int64_t orc_sample_rows(const int64_t *indptr, const int32_t *indices, const int32_t *dst_nodes,
                        int32_t n_dst, int32_t fanout, uint64_t seed, uint32_t step, uint32_t layer,
                        int32_t *b_indptr, int32_t *e_glob)
{
    int64_t *pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)(fanout > 0 ? fanout : 1));
    int64_t nnz = 0;
    b_indptr[0] = 0;
    for (int32_t i = 0; i < n_dst; ++i) {
        int32_t v = dst_nodes[i];
        int64_t start = indptr[v], d = indptr[v + 1] - start;
        int32_t m = orc_sample_positions(d, fanout, seed, step, layer, (uint32_t)v, pos);
        for (int32_t t = 0; t < m; ++t) e_glob[nnz + t] = indices[start + pos[t]];
        nnz += m;
        b_indptr[i + 1] = (int32_t)nnz;
    }
    free(pos);
    return nnz;
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Source frontier of a block: the destination nodes first, in their given
 * order, then every sampled node that is not a destination, each once, in
 * ascending global id.  b_cols[e] is the index of e_glob[e] in src_nodes.
 * Returns n_src.                                                          */
int32_t orc_build_frontier(int64_t n_nodes, const int32_t *dst_nodes, int32_t n_dst,
                           const int32_t *e_glob, int64_t nnz, int32_t *src_nodes, int32_t *b_cols)
{
    int32_t *local = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_nodes);
    for (int64_t v = 0; v < n_nodes; ++v) local[v] = -1;
    for (int32_t i = 0; i < n_dst; ++i) { local[dst_nodes[i]] = i; src_nodes[i] = dst_nodes[i]; }
    int32_t n_new = 0;
    for (int64_t e = 0; e < nnz; ++e) {
        int32_t g = e_glob[e];
        if (local[g] == -1) { local[g] = -2; src_nodes[n_dst + n_new++] = g; }
    }
    qsort(src_nodes + n_dst, (size_t)n_new, sizeof(int32_t), cmp_i32);
    for (int32_t r = 0; r < n_new; ++r) local[src_nodes[n_dst + r]] = n_dst + r;
    for (int64_t e = 0; e < nnz; ++e) b_cols[e] = local[e_glob[e]];
    free(local);
    return n_dst + n_new;
}

/* Transposed block: for each source j the destinations that sampled it,
 * ascending (stable counting sort of the edges by column).               */
void orc_transpose_block(int32_t n_dst, int32_t n_src, const int32_t *b_indptr, const int32_t *b_cols,
                         int32_t *t_indptr, int32_t *t_rows)
{
    int32_t nnz = b_indptr[n_dst];
    for (int32_t j = 0; j <= n_src; ++j) t_indptr[j] = 0;
    for (int32_t e = 0; e < nnz; ++e) t_indptr[b_cols[e] + 1]++;
    for (int32_t j = 0; j < n_src; ++j) t_indptr[j + 1] += t_indptr[j];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_src > 0 ? n_src : 1));
    for (int32_t j = 0; j < n_src; ++j) cursor[j] = t_indptr[j];
    for (int32_t i = 0; i < n_dst; ++i)
        for (int32_t e = b_indptr[i]; e < b_indptr[i + 1]; ++e) t_rows[cursor[b_cols[e]]++] = i;
    free(cursor);
}

/* out[j, :] = X[idx[j], :], a copy of row_bytes bytes per row.          */
void orc_gather_rows(const void *X, int64_t ldx_bytes, int64_t row_bytes, const int32_t *idx, int64_t n,
                     void *out, int64_t ldo_bytes)
{
    for (int64_t j = 0; j < n; ++j)
        memcpy((char *)out + j * ldo_bytes, (const char *)X + (int64_t)idx[j] * ldx_bytes, (size_t)row_bytes);
}

/* Mean aggregation: A[i,:] = (1/m_i) * sum over the row's edges of H[col,:],
 * m_i = number of edges of row i; a row without edges gives zeros.  An edge
 * listed twice counts twice.  indptr is int64 so a whole graph also fits. */
void orc_aggregate_fwd(int64_t n_dst, const int64_t *b_indptr, const int32_t *b_cols, const double *H,
                       int64_t F, double *A)
{
    for (int64_t i = 0; i < n_dst; ++i) {
        double *a = A + i * F;
        for (int64_t f = 0; f < F; ++f) a[f] = 0.0;
        int64_t m = b_indptr[i + 1] - b_indptr[i];
        if (m == 0) continue;
        for (int64_t e = b_indptr[i]; e < b_indptr[i + 1]; ++e) {
            const double *h = H + (int64_t)b_cols[e] * F;
            for (int64_t f = 0; f < F; ++f) a[f] += h[f];
        }
        for (int64_t f = 0; f < F; ++f) a[f] /= (double)m;
    }
}

/* GraphSAGE-mean projection: Z = Hself*W[0:in,:] + A*W[in:2in,:] + b,
 * Y = max(Z,0) if relu else Z.  W is [2*in, out] row-major.              */
void orc_linear_fwd(int64_t n, int64_t in, int64_t out, const double *Hself, int64_t ldh, const double *A,
                    const double *W, const double *b, int32_t relu, double *Y)
{
    for (int64_t i = 0; i < n; ++i)
        for (int64_t o = 0; o < out; ++o) {
            double z = b[o];
            for (int64_t k = 0; k < in; ++k) z += Hself[i * ldh + k] * W[k * out + o];
            for (int64_t k = 0; k < in; ++k) z += A[i * in + k] * W[(in + k) * out + o];
            Y[i * out + o] = (relu && !(z > 0.0)) ? 0.0 : z;
        }
}

/* Softmax cross-entropy, mean over the batch:
 * loss = (1/B) sum_i [log sum_c exp(Z[i,c]) - Z[i,y_i]],
 * dZ = (softmax(Z) - onehot(y)) / B.                                      */
double orc_softmax_xent(int64_t B, int64_t C, const double *Z, const int32_t *y, double *dZ)
{
    double loss = 0.0;
    for (int64_t i = 0; i < B; ++i) {
        const double *z = Z + i * C;
        double zmax = z[0];
        for (int64_t c = 1; c < C; ++c) if (z[c] > zmax) zmax = z[c];
        double s = 0.0;
        for (int64_t c = 0; c < C; ++c) s += exp(z[c] - zmax);
        loss += log(s) + zmax - z[y[i]];
        if (dZ)
            for (int64_t c = 0; c < C; ++c)
                dZ[i * C + c] = (exp(z[c] - zmax) / s - (c == y[i] ? 1.0 : 0.0)) / (double)B;
    }
    return loss / (double)B;
}

/* Backward of the projection.  dZ = dY masked by Y > 0 when relu (strictly
 * positive: the derivative at 0 is taken as 0).  dW = [Hself|A]^T dZ,
 * db = column sums of dZ, dSelf = dZ W_self^T, dAgg = dZ W_neigh^T
 * (dSelf/dAgg may be NULL).  dZ_out (nullable) receives the masked dZ.    */
void orc_linear_bwd(int64_t n, int64_t in, int64_t out, const double *dY, const double *Y, int32_t relu,
                    const double *Hself, int64_t ldh, const double *A, const double *W, double *dW,
                    double *db, double *dSelf, double *dAgg)
{
    double *dZ = (double *)malloc(sizeof(double) * (size_t)(n * out > 0 ? n * out : 1));
    for (int64_t i = 0; i < n * out; ++i) dZ[i] = (relu && !(Y[i] > 0.0)) ? 0.0 : dY[i];
    for (int64_t k = 0; k < 2 * in * out; ++k) dW[k] = 0.0;
    for (int64_t o = 0; o < out; ++o) db[o] = 0.0;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t o = 0; o < out; ++o) {
            double g = dZ[i * out + o];
            db[o] += g;
            for (int64_t k = 0; k < in; ++k) {
                dW[k * out + o] += Hself[i * ldh + k] * g;
                dW[(in + k) * out + o] += A[i * in + k] * g;
            }
        }
    if (dSelf && dAgg)
        for (int64_t i = 0; i < n; ++i)
            for (int64_t k = 0; k < in; ++k) {
                double s = 0.0, a = 0.0;
                for (int64_t o = 0; o < out; ++o) {
                    s += dZ[i * out + o] * W[k * out + o];
                    a += dZ[i * out + o] * W[(in + k) * out + o];
                }
                dSelf[i * in + k] = s;
                dAgg[i * in + k] = a;
            }
    free(dZ);
}

/* Backward of the mean aggregation plus the self path:
 * dH[j,:] = [j < n_dst] dSelf[j,:] + sum over edges (i -> j) dAgg[i,:]/m_i. */
void orc_aggregate_bwd(int64_t n_dst, int64_t n_src, const int64_t *b_indptr, const int32_t *b_cols,
                       const double *dAgg, const double *dSelf, int64_t F, double *dH)
{
    for (int64_t j = 0; j < n_src; ++j)
        for (int64_t f = 0; f < F; ++f) dH[j * F + f] = (dSelf && j < n_dst) ? dSelf[j * F + f] : 0.0;
    for (int64_t i = 0; i < n_dst; ++i) {
        int64_t m = b_indptr[i + 1] - b_indptr[i];
        for (int64_t e = b_indptr[i]; e < b_indptr[i + 1]; ++e)
            for (int64_t f = 0; f < F; ++f) dH[(int64_t)b_cols[e] * F + f] += dAgg[i * F + f] / (double)m;
    }
}

/* GCN aggregation on a sampled block (Sec. III-E lists GCN among the integrated models):
 * A[i,:] = s[i] * sum over the row's edges of c[col] * H[col,:]  +  selfw[i] * H[i,:].
 * s, selfw are per destination row, c per source row (see gcn_weights in the Python part). */
void orc_gcn_aggregate_fwd(int64_t n_dst, const int64_t *b_indptr, const int32_t *b_cols, const double *H,
                           int64_t F, const double *s, const double *c, const double *selfw, double *A)
{
    for (int64_t i = 0; i < n_dst; ++i) {
        double *a = A + i * F;
        for (int64_t f = 0; f < F; ++f) a[f] = 0.0;
        for (int64_t e = b_indptr[i]; e < b_indptr[i + 1]; ++e) {
            const double *h = H + (int64_t)b_cols[e] * F;
            const double w = c[b_cols[e]];
            for (int64_t f = 0; f < F; ++f) a[f] += w * h[f];
        }
        for (int64_t f = 0; f < F; ++f) a[f] = s[i] * a[f] + selfw[i] * H[i * F + f];
    }
}

/* Its transpose: dH[j,:] = c[j] * sum over edges (i -> j) of s[i] * dA[i,:]  +  [j < n_dst] selfw[j] * dA[j,:]. */
void orc_gcn_aggregate_bwd(int64_t n_dst, int64_t n_src, const int64_t *b_indptr, const int32_t *b_cols,
                           const double *dA, int64_t F, const double *s, const double *c, const double *selfw,
                           double *dH)
{
    for (int64_t j = 0; j < n_src; ++j)
        for (int64_t f = 0; f < F; ++f) dH[j * F + f] = 0.0;
    for (int64_t i = 0; i < n_dst; ++i)
        for (int64_t e = b_indptr[i]; e < b_indptr[i + 1]; ++e)
            for (int64_t f = 0; f < F; ++f) dH[(int64_t)b_cols[e] * F + f] += s[i] * dA[i * F + f];
    for (int64_t j = 0; j < n_src; ++j)
        for (int64_t f = 0; f < F; ++f) {
            dH[j * F + f] *= c[j];
            if (j < n_dst) dH[j * F + f] += selfw[j] * dA[j * F + f];
        }
}

/* Plain SGD: w <- w - lr * g.                                           */
void orc_sgd(int64_t n, double *w, const double *g, double lr)
{
    for (int64_t i = 0; i < n; ++i) w[i] -= lr * g[i];
}

/* Round each value to the nearest bfloat16 (8-bit exponent, 7-bit
 * mantissa), ties to even, and return it as a double.  Used at the points
 * where the bf16 configuration stores a tensor.                          */
void orc_round_bf16(int64_t n, double *x)
{
    for (int64_t i = 0; i < n; ++i) {
        double v = x[i];
        if (v == 0.0 || isnan(v) || isinf(v)) continue;
        int e;
        double frac = frexp(v, &e);              /* v = frac * 2^e, 0.5 <= |frac| < 1 */
        if (e - 1 < -126) {                      /* below the normal range: fixed spacing 2^-133 */
            double q = ldexp(1.0, -133);
            x[i] = nearbyint(v / q) * q;
            continue;
        }
        double scaled = ldexp(frac, 8);          /* 8 significant bits: 128 <= |scaled| < 256 */
        x[i] = ldexp(nearbyint(scaled), e - 8);  /* nearbyint: ties to even in the default mode */
    }
}
