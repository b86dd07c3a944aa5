/*
 * CPU oracle for one TMA trainer's local training path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what
 * the GPU library computes.  It shares no code, header, table or helper with
 * the HIP sources; nothing in the product path may call it.  Only the test
 * suite, the smoke check and the benchmark's CPU-baseline leg load it.
 *
 * Everything floating point is fp64, single-threaded, written as the
 * definition reads: adjacency scanned entry by entry, matrix products as
 * triple loops, no blocking, no fusion.
 * For the benchmark's all-cores timing leg only, orc_set_threads(n > 1) lets
 * the row loops of the aggregation and of the SAGE layer (the ones whose
 * iterations are independent, or plain sums over rows) run under an OpenMP
 * parallel-for: the same loops, split over rows.  Every test runs with the
 * default of one thread, where those pragmas are inactive.
 *
 * Passages of the paper each function follows are named in its comment
 * (Preliminaries = the paragraph defining alpha, alpha^-1 and the node-induced
 * subgraph; Sec. 3.2.2 = the two randomized partition schemes; Thm. 1 and its
 * proof in App. B = the row-normalised one-layer model, its L2 loss and the
 * chain rule; Alg. 1/2 = server and trainer loops).
 *
 * Pins (see tests/test_oracle_*.py): published SplitMix64 test vector,
 * partition invariants and the 1/M kept-edge ratio the paper prints, brute
 * force edge filtering, dense-matrix products, the closed-form initial
 * gradient from the proof of Thm. 1, the expected neighbour mean
 * [(1-h), h], central finite differences and the adjoint identity.
 * The composed multi-layer training step has no value printed in the paper:
 * it is pinned only through its parts plus finite differences.
 * GCN and dense layers (tests/test_oracle_gcn.py): the sqrt-degree eigenvector
 * of the normalised adjacency, its forms on regular, complete and empty graphs,
 * a sparse library's matrix algebra, a library's reverse-mode derivative, the
 * adjoint identity and finite differences.
 * Link-prediction head (tests/test_oracle_link.py): membership of every drawn
 * positive in the edge list, tail != positive tail, chi-square uniformity of
 * both draws, a library's index / multiply / PReLU / BCE routines with their
 * reverse-mode derivatives, finite differences through encoder + decoder.
 */
#include <math.h>
#include <omp.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

static int orc_nthreads = 1;
void orc_set_threads(int n) { orc_nthreads = n < 1 ? 1 : n; }
int orc_hardware_threads(void) { return omp_get_num_procs(); }
#define ORC_ROWS _Pragma("omp parallel for schedule(static) num_threads(orc_nthreads) if(orc_nthreads > 1)")

/* ------------------------------------------------------------------------
 * Random assignment (Sec. 3.2.2): every node, or every super-node, goes
 * independently and uniformly to one of K partitions.  The paper fixes no
 * generator; this build's written spec is
 *     z    = SplitMix64 output number (id+1) of the stream seeded with `seed`
 *     part = floor(z * K / 2^64)
 * SplitMix64 (Steele, Lea, Flood 2014): state += 0x9E3779B97F4A7C15 per draw,
 * output = finaliser(state).
 * ---------------------------------------------------------------------- */
uint64_t orc_mix64(uint64_t seed, uint64_t id)
{
    uint64_t z = seed + (id + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static int32_t uniform_k(uint64_t seed, uint64_t id, int32_t K)
{
    unsigned __int128 wide = (unsigned __int128)orc_mix64(seed, id) * (uint64_t)K;
    return (int32_t)(wide >> 64);
}

/* cluster == NULL: RandomTMA, the unit of randomness is the node.
 * cluster != NULL: SuperTMA, the unit is the super-node cluster[v]; a node
 * inherits the partition of its super-node. */
void orc_partition(int64_t n_nodes, const int32_t *cluster, int32_t K,
                   uint64_t seed, int32_t *part)
{
    for (int64_t v = 0; v < n_nodes; ++v) {
        uint64_t unit = cluster ? (uint64_t)cluster[v] : (uint64_t)v;
        part[v] = uniform_k(seed, unit, K);
    }
}

/* ------------------------------------------------------------------------
 * Node-induced subgraph of partition p (Preliminaries):
 *   V^(p) = { v : part[v] = p },  E^(p) = { (u,v) in E : u, v in V^(p) }.
 * Canonical form so that the result is unique: local id = rank of the global
 * id inside V^(p); neighbours keep the order of the input row.
 * ---------------------------------------------------------------------- */
void orc_induced_count(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx,
                       const int32_t *part, int32_t p,
                       int64_t *n_loc, int64_t *nnz_loc)
{
    int64_t nl = 0, el = 0;
    for (int64_t v = 0; v < n_nodes; ++v) {
        if (part[v] != p) continue;
        ++nl;
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e)
            if (part[colidx[e]] == p) ++el;
    }
    *n_loc = nl;
    *nnz_loc = el;
}

void orc_induced_fill(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx,
                      const int32_t *part, int32_t p,
                      int32_t *g2l,        /* [n_nodes], -1 outside the part */
                      int32_t *l2g,        /* [n_loc] */
                      int32_t *rowptr_loc, /* [n_loc+1] */
                      int32_t *colidx_loc, /* [nnz_loc] */
                      double *inv_deg)     /* [n_loc], 0 for isolated nodes */
{
    int32_t nl = 0;
    for (int64_t v = 0; v < n_nodes; ++v) {
        if (part[v] == p) { g2l[v] = nl; l2g[nl] = (int32_t)v; ++nl; }
        else g2l[v] = -1;
    }
    int32_t el = 0;
    rowptr_loc[0] = 0;
    for (int32_t i = 0; i < nl; ++i) {
        int64_t v = l2g[i];
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            int32_t u = colidx[e];
            if (part[u] == p) colidx_loc[el++] = g2l[u];
        }
        rowptr_loc[i + 1] = el;
        int32_t d = rowptr_loc[i + 1] - rowptr_loc[i];
        inv_deg[i] = d > 0 ? 1.0 / (double)d : 0.0;
    }
}

/* ------------------------------------------------------------------------
 * Mean aggregation with the row-normalised adjacency (Thm. 1 and the first
 * equation of its proof): m_v = sum_{u in N'(v)} x_u / d_v, over the
 * effective (local) neighbourhood.  A node with no local neighbour gets 0.
 * ---------------------------------------------------------------------- */
void orc_mean_aggregate(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                        const double *H, int64_t F, double *M)
{
    ORC_ROWS
    for (int64_t v = 0; v < n; ++v) {
        double *m = M + v * F;
        for (int64_t f = 0; f < F; ++f) m[f] = 0.0;
        int32_t d = rowptr[v + 1] - rowptr[v];
        if (d == 0) continue;
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            const double *h = H + (int64_t)colidx[e] * F;
            for (int64_t f = 0; f < F; ++f) m[f] += h[f];
        }
        for (int64_t f = 0; f < F; ++f) m[f] /= (double)d;
    }
}

/* Transposed operator: out = Abar^T G, i.e. every entry (v,u) of the CSR
 * sends G_v / d_v to row u.  Written as a scatter so that it does not rely on
 * the graph being symmetric. */
void orc_mean_aggregate_T(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                          const double *G, int64_t F, double *out)
{
    memset(out, 0, (size_t)(n * F) * sizeof(double));
    for (int64_t v = 0; v < n; ++v) {
        int32_t d = rowptr[v + 1] - rowptr[v];
        if (d == 0) continue;
        const double *g = G + v * F;
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            double *o = out + (int64_t)colidx[e] * F;
            for (int64_t f = 0; f < F; ++f) o[f] += g[f] / (double)d;
        }
    }
}

/* ------------------------------------------------------------------------
 * One mean-aggregation GraphSAGE layer.  The paper names the encoder and, in
 * Thm. 1, writes its aggregation as Abar X W; the layer used here is
 *     M = Abar H,  Z = H W_self + M W_neigh + 1 b^T,  H' = act(Z)
 * with act = identity (0) or ReLU (1).  W_* are [F_in, F_out] row-major.
 * ---------------------------------------------------------------------- */
void orc_sage_layer_fwd(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                        const double *H, int64_t F_in,
                        const double *W_self, const double *W_neigh, const double *bias,
                        int64_t F_out, int act,
                        double *M, double *Z, double *Hnext)
{
    orc_mean_aggregate(n, rowptr, colidx, H, F_in, M);
    ORC_ROWS
    for (int64_t v = 0; v < n; ++v) {
        double *z = Z + v * F_out;
        for (int64_t o = 0; o < F_out; ++o) z[o] = bias[o];
        for (int64_t k = 0; k < F_in; ++k) {
            double h = H[v * F_in + k], m = M[v * F_in + k];
            for (int64_t o = 0; o < F_out; ++o)
                z[o] += h * W_self[k * F_out + o] + m * W_neigh[k * F_out + o];
        }
        for (int64_t o = 0; o < F_out; ++o)
            Hnext[v * F_out + o] = (act == 1) ? (z[o] > 0.0 ? z[o] : 0.0) : z[o];
    }
}

/* Chain rule through the layer (the proof of Thm. 1 writes the one-layer
 * instance: dL/dw = dL/dz * dz/dg * dg/dw):
 *   dZ = dH' (.) act'(Z)
 *   dW_self = H^T dZ,  dW_neigh = M^T dZ,  db = column sums of dZ
 *   dH = dZ W_self^T + Abar^T (dZ W_neigh^T)        (skipped when dH == NULL)
 * scratch: n*F_in doubles. */
void orc_sage_layer_bwd(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                        const double *H, const double *M, const double *Z,
                        const double *dHnext,
                        const double *W_self, const double *W_neigh,
                        int64_t F_in, int64_t F_out, int act,
                        double *dW_self, double *dW_neigh, double *dbias,
                        double *dH, double *scratch_dM, double *scratch_dZ)
{
    double *dZ = scratch_dZ;
    for (int64_t i = 0; i < n * F_out; ++i)
        dZ[i] = (act == 1) ? (Z[i] > 0.0 ? dHnext[i] : 0.0) : dHnext[i];

    for (int64_t i = 0; i < F_in * F_out; ++i) dW_self[i] = dW_neigh[i] = 0.0;
    for (int64_t o = 0; o < F_out; ++o) dbias[o] = 0.0;
    const int64_t nW = F_in * F_out;
#pragma omp parallel for schedule(static) num_threads(orc_nthreads) if(orc_nthreads > 1) \
    reduction(+ : dW_self[:nW], dW_neigh[:nW], dbias[:F_out])
    for (int64_t v = 0; v < n; ++v) {       /* sums over nodes, one node at a time */
        const double *g = dZ + v * F_out;
        for (int64_t k = 0; k < F_in; ++k) {
            double h = H[v * F_in + k], m = M[v * F_in + k];
            for (int64_t o = 0; o < F_out; ++o) {
                dW_self[k * F_out + o] += h * g[o];
                dW_neigh[k * F_out + o] += m * g[o];
            }
        }
        for (int64_t o = 0; o < F_out; ++o) dbias[o] += g[o];
    }
    if (!dH) return;

    double *dM = scratch_dM;
    ORC_ROWS
    for (int64_t v = 0; v < n; ++v)
        for (int64_t k = 0; k < F_in; ++k) {
            double s = 0.0, t = 0.0;
            for (int64_t o = 0; o < F_out; ++o) {
                s += dZ[v * F_out + o] * W_self[k * F_out + o];
                t += dZ[v * F_out + o] * W_neigh[k * F_out + o];
            }
            dH[v * F_in + k] = s;
            dM[v * F_in + k] = t;
        }
    /* dH += Abar^T dM, as a scatter */
    for (int64_t v = 0; v < n; ++v) {
        int32_t d = rowptr[v + 1] - rowptr[v];
        if (d == 0) continue;
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            double *o = dH + (int64_t)colidx[e] * F_in;
            for (int64_t k = 0; k < F_in; ++k) o[k] += dM[v * F_in + k] / (double)d;
        }
    }
}

/* ------------------------------------------------------------------------
 * Losses.
 * Softmax cross-entropy, mean over the n local nodes (this build's reading
 * for workloads that carry class labels; the paper's own task head is out of
 * scope).  dlogits = (softmax - onehot) / n.
 * ---------------------------------------------------------------------- */
double orc_softmax_ce(int64_t n, int64_t C, const double *logits,
                      const int32_t *labels, double *dlogits)
{
    double loss = 0.0;
    for (int64_t v = 0; v < n; ++v) {
        const double *z = logits + v * C;
        double mx = z[0];
        for (int64_t c = 1; c < C; ++c) if (z[c] > mx) mx = z[c];
        double se = 0.0;
        for (int64_t c = 0; c < C; ++c) se += exp(z[c] - mx);
        double lse = mx + log(se);
        loss += lse - z[labels[v]];
        if (dlogits)
            for (int64_t c = 0; c < C; ++c)
                dlogits[v * C + c] =
                    (exp(z[c] - lse) - (c == labels[v] ? 1.0 : 0.0)) / (double)n;
    }
    return loss / (double)n;
}

/* The loss of Thm. 1: z = sigmoid(g), L = 1/2 ||y - z||^2 summed over nodes
 * and outputs; dL/dg = (z - y) z (1 - z)  (proof of Thm. 1, gradient
 * equations). */
double orc_sigmoid_l2(int64_t n, int64_t C, const double *G, const double *Y, double *dG)
{
    double loss = 0.0;
    for (int64_t i = 0; i < n * C; ++i) {
        double z = 1.0 / (1.0 + exp(-G[i]));
        double r = z - Y[i];
        loss += 0.5 * r * r;
        if (dG) dG[i] = r * z * (1.0 - z);
    }
    return loss;
}

/* ------------------------------------------------------------------------
 * Normalisation and activation of the paper's encoders (Sec. 4.1, paragraph
 * on GNN encoders: PReLU as non-linearity, Layer Normalization before the
 * activation), applied to a layer's pre-activation Z [n, F]:
 *     mu_v  = mean_f Z_vf,  var_v = mean_f (Z_vf - mu_v)^2      (per node)
 *     Zh    = (Z - mu) / sqrt(var + eps)
 *     Y     = gamma (.) Zh + beta
 *     H'    = Y            where Y > 0
 *             slope * Y    elsewhere                              (PReLU)
 * The paper gives no more than the two names; readings taken here: the
 * normalisation runs over the feature axis of each node with a learnable
 * scale and shift per feature and the biased variance (Ba et al. 2016), the
 * activation has ONE learnable slope per layer (He et al. 2015, shared
 * variant).  `open` (optional, n*F bytes) overrides the decision Y > 0 in the
 * backward pass, as for ReLU.
 * ---------------------------------------------------------------------- */
void orc_layernorm_prelu_fwd(int64_t n, int64_t F, const double *Z, const double *gamma,
                             const double *beta, double slope, double eps, double *Hn)
{
    for (int64_t v = 0; v < n; ++v) {
        const double *z = Z + v * F;
        double mu = 0.0;
        for (int64_t f = 0; f < F; ++f) mu += z[f];
        mu /= (double)F;
        double var = 0.0;
        for (int64_t f = 0; f < F; ++f) var += (z[f] - mu) * (z[f] - mu);
        var /= (double)F;
        const double rstd = 1.0 / sqrt(var + eps);
        for (int64_t f = 0; f < F; ++f) {
            const double y = gamma[f] * ((z[f] - mu) * rstd) + beta[f];
            Hn[v * F + f] = y > 0.0 ? y : slope * y;
        }
    }
}

/* Chain rule through the three maps above.  With Zh, Y as in the forward pass and g = dL/dH':
 *     dY      = g            where Y > 0,   slope * g elsewhere
 *     dslope  = sum over all v,f with Y <= 0 of g * Y
 *     dgamma_f = sum_v dY_vf Zh_vf,   dbeta_f = sum_v dY_vf
 *     dZh     = dY (.) gamma
 *     dZ_v    = ( dZh_v - mean_f(dZh_v) - Zh_v * mean_f(dZh_v (.) Zh_v) ) / sqrt(var_v + eps)
 */
void orc_layernorm_prelu_bwd(int64_t n, int64_t F, const double *Z, const double *dHn,
                             const double *gamma, const double *beta, double slope, double eps,
                             const uint8_t *open, double *dZ, double *dgamma, double *dbeta,
                             double *dslope, double *zh, double *dzh)
{
    for (int64_t f = 0; f < F; ++f) { dgamma[f] = 0.0; dbeta[f] = 0.0; }
    double ds = 0.0;
    for (int64_t v = 0; v < n; ++v) {
        const double *z = Z + v * F;
        double mu = 0.0;
        for (int64_t f = 0; f < F; ++f) mu += z[f];
        mu /= (double)F;
        double var = 0.0;
        for (int64_t f = 0; f < F; ++f) var += (z[f] - mu) * (z[f] - mu);
        var /= (double)F;
        const double rstd = 1.0 / sqrt(var + eps);
        double m1 = 0.0, m2 = 0.0;
        for (int64_t f = 0; f < F; ++f) {
            zh[f] = (z[f] - mu) * rstd;
            const double y = gamma[f] * zh[f] + beta[f];
            const double g = dHn[v * F + f];
            const int is_open = open ? (open[v * F + f] != 0) : (y > 0.0);
            const double dy = is_open ? g : slope * g;
            if (!is_open) ds += g * y;
            dgamma[f] += dy * zh[f];
            dbeta[f] += dy;
            dzh[f] = dy * gamma[f];
            m1 += dzh[f];
            m2 += dzh[f] * zh[f];
        }
        m1 /= (double)F;
        m2 /= (double)F;
        for (int64_t f = 0; f < F; ++f) dZ[v * F + f] = (dzh[f] - m1 - zh[f] * m2) * rstd;
    }
    *dslope = ds;
}

/* ------------------------------------------------------------------------
 * Optimizer step (Alg. 2, the `optimizer` call; read as plain SGD) and the
 * aggregation operator phi = arithmetic mean of the trainers' parameters
 * (Sec. 3.1; Alg. 1 aggregation line), followed by the overwrite of every
 * participating trainer's weights (Alg. 2).  Trainers whose bit in `active`
 * is clear take no part and are left untouched (failure experiment, Sec. 4.4).
 * W is [M][P] row-major.
 * ---------------------------------------------------------------------- */
void orc_sgd_step(int64_t P, double *W, const double *dW, double lr)
{
    for (int64_t i = 0; i < P; ++i) W[i] -= lr * dW[i];
}

/* Adam (Kingma & Ba 2015) as a second choice for Alg. 2's `optimizer` call, which the paper leaves
 * unnamed.  t = 1, 2, ... is the number of the step being taken.  The moment estimates m, v are the
 * trainer's own state: the aggregation operator averages model parameters only (Sec. 3.1).
 *     m <- b1 m + (1-b1) g,   v <- b2 v + (1-b2) g^2,
 *     W <- W - lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)                                    */
void orc_adam_step(int64_t P, double *W, const double *dW, double *m, double *v, double lr,
                   double b1, double b2, double eps, int64_t t)
{
    const double c1 = 1.0 - pow(b1, (double)t), c2 = 1.0 - pow(b2, (double)t);
    for (int64_t i = 0; i < P; ++i) {
        m[i] = b1 * m[i] + (1.0 - b1) * dW[i];
        v[i] = b2 * v[i] + (1.0 - b2) * dW[i] * dW[i];
        W[i] -= lr * (m[i] / c1) / (sqrt(v[i] / c2) + eps);
    }
}

void orc_average(int32_t M, int64_t P, uint64_t active, double *W, double *W_global)
{
    int cnt = 0;
    for (int32_t i = 0; i < M; ++i) if ((active >> i) & 1u) ++cnt;
    if (cnt == 0) return;
    for (int64_t j = 0; j < P; ++j) {
        double s = 0.0;
        for (int32_t i = 0; i < M; ++i)
            if ((active >> i) & 1u) s += W[(int64_t)i * P + j];
        s /= (double)cnt;
        if (W_global) W_global[j] = s;
        for (int32_t i = 0; i < M; ++i)
            if ((active >> i) & 1u) W[(int64_t)i * P + j] = s;
    }
}

/* ------------------------------------------------------------------------
 * Other encoders of Sec. 4.1 (paragraph on GNN encoders): the graph
 * convolution of Kipf & Welling (2017), which the paper cites for its GCN
 * encoder, and the graph-agnostic MLP encoder.
 *
 * GCN layer on the local (node-induced) subgraph:
 *     Ahat = Dt^-1/2 (A + I) Dt^-1/2,   Dt = diag(d_v + 1)   (d_v = local degree)
 *     M = Ahat H,   Z = M W + 1 b^T,   H' = act(Z)
 * Entry (v,u) of Ahat is s_v s_u for every CSR entry (v,u) plus s_v^2 on the
 * diagonal, with s_v = (d_v + 1)^-1/2.  The degree on both sides is the row's
 * own entry count; the local graphs here store both directions of every edge,
 * so this is the symmetric normalisation of the cited paper.
 * ---------------------------------------------------------------------- */
void orc_gcn_norm(int64_t n, const int32_t *rowptr, double *s)
{
    for (int64_t v = 0; v < n; ++v) s[v] = 1.0 / sqrt((double)(rowptr[v + 1] - rowptr[v]) + 1.0);
}

void orc_gcn_aggregate(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                       const double *H, int64_t F, double *M)
{
    for (int64_t v = 0; v < n; ++v) {
        const double sv = 1.0 / sqrt((double)(rowptr[v + 1] - rowptr[v]) + 1.0);
        double *m = M + v * F;
        for (int64_t f = 0; f < F; ++f) m[f] = sv * sv * H[v * F + f];
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            const int64_t u = colidx[e];
            const double su = 1.0 / sqrt((double)(rowptr[u + 1] - rowptr[u]) + 1.0);
            for (int64_t f = 0; f < F; ++f) m[f] += sv * su * H[u * F + f];
        }
    }
}

/* out = Ahat^T G as a scatter over the same CSR (no symmetry assumed). */
void orc_gcn_aggregate_T(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                         const double *G, int64_t F, double *out)
{
    memset(out, 0, (size_t)(n * F) * sizeof(double));
    for (int64_t v = 0; v < n; ++v) {
        const double sv = 1.0 / sqrt((double)(rowptr[v + 1] - rowptr[v]) + 1.0);
        for (int64_t f = 0; f < F; ++f) out[v * F + f] += sv * sv * G[v * F + f];
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            const int64_t u = colidx[e];
            const double su = 1.0 / sqrt((double)(rowptr[u + 1] - rowptr[u]) + 1.0);
            for (int64_t f = 0; f < F; ++f) out[u * F + f] += sv * su * G[v * F + f];
        }
    }
}

/* Z = X W + 1 b^T (b may be NULL), Y = act(Z): the MLP encoder's layer, the
 * transform of the GCN layer (X = Ahat H) and, without bias, a layer of the
 * link decoder (App., formulation of the MLP decoder). */
void orc_dense_fwd(int64_t n, const double *X, int64_t F_in, const double *W, const double *bias,
                   int64_t F_out, int act, double *Z, double *Y)
{
    for (int64_t v = 0; v < n; ++v) {
        double *z = Z + v * F_out;
        for (int64_t o = 0; o < F_out; ++o) z[o] = bias ? bias[o] : 0.0;
        for (int64_t k = 0; k < F_in; ++k) {
            const double x = X[v * F_in + k];
            for (int64_t o = 0; o < F_out; ++o) z[o] += x * W[k * F_out + o];
        }
        for (int64_t o = 0; o < F_out; ++o)
            Y[v * F_out + o] = (act == 1) ? (z[o] > 0.0 ? z[o] : 0.0) : z[o];
    }
}

/* dZ = dY (.) act'(Z);  dW = X^T dZ;  db = column sums of dZ (skipped when NULL);
 * dX = dZ W^T (skipped when NULL).  scratch_dZ: n*F_out doubles. */
void orc_dense_bwd(int64_t n, const double *X, const double *Z, const double *dY, const double *W,
                   int64_t F_in, int64_t F_out, int act, double *dW, double *dbias, double *dX,
                   double *scratch_dZ)
{
    double *dZ = scratch_dZ;
    for (int64_t i = 0; i < n * F_out; ++i)
        dZ[i] = (act == 1) ? (Z[i] > 0.0 ? dY[i] : 0.0) : dY[i];
    for (int64_t i = 0; i < F_in * F_out; ++i) dW[i] = 0.0;
    if (dbias) for (int64_t o = 0; o < F_out; ++o) dbias[o] = 0.0;
    for (int64_t v = 0; v < n; ++v) {
        for (int64_t k = 0; k < F_in; ++k)
            for (int64_t o = 0; o < F_out; ++o) dW[k * F_out + o] += X[v * F_in + k] * dZ[v * F_out + o];
        if (dbias) for (int64_t o = 0; o < F_out; ++o) dbias[o] += dZ[v * F_out + o];
    }
    if (!dX) return;
    for (int64_t v = 0; v < n; ++v)
        for (int64_t k = 0; k < F_in; ++k) {
            double s = 0.0;
            for (int64_t o = 0; o < F_out; ++o) s += dZ[v * F_out + o] * W[k * F_out + o];
            dX[v * F_in + k] = s;
        }
}

void orc_gcn_layer_fwd(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                       const double *H, int64_t F_in, const double *W, const double *bias,
                       int64_t F_out, int act, double *M, double *Z, double *Hnext)
{
    orc_gcn_aggregate(n, rowptr, colidx, H, F_in, M);
    orc_dense_fwd(n, M, F_in, W, bias, F_out, act, Z, Hnext);
}

/* dW = M^T dZ, db = 1^T dZ, dH = Ahat^T (dZ W^T)   (dH skipped when NULL).
 * scratch_dM: n*F_in doubles, scratch_dZ: n*F_out doubles. */
void orc_gcn_layer_bwd(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                       const double *M, const double *Z, const double *dHnext, const double *W,
                       int64_t F_in, int64_t F_out, int act, double *dW, double *dbias, double *dH,
                       double *scratch_dM, double *scratch_dZ)
{
    orc_dense_bwd(n, M, Z, dHnext, W, F_in, F_out, act, dW, dbias, dH ? scratch_dM : NULL, scratch_dZ);
    if (dH) orc_gcn_aggregate_T(n, rowptr, colidx, scratch_dM, F_in, dH);
}

/* ------------------------------------------------------------------------
 * GCN layer on one bipartite block of a sampled message-flow graph (Sec. 4.1:
 * the GCN encoder is trained with the neighbour sampler on the larger
 * datasets).  A block has n_dst rows over n_src >= n_dst source nodes, the
 * destination nodes being the first n_dst sources.  The symmetric
 * normalisation of the full-graph layer needs a degree for the source side,
 * which a sampled block does not define (how often a source was drawn depends
 * on which destinations were asked).  Reading taken here: the row-normalised
 * form with the self-loop,
 *     m_v = ( h_v + sum_{u in S(v)} h_u ) / ( |S(v)| + 1 ),   Z = M W + 1 b^T,
 * i.e. Dt^-1 (A_S + I): the mean over the sampled neighbourhood and the node
 * itself, which is how the cited neighbour-sampling method writes its GCN
 * variant.  With S(v) = N(v) it is the random-walk normalisation of A + I.
 * ---------------------------------------------------------------------- */
void orc_gcn_block_aggregate(int64_t n_dst, const int32_t *rowptr, const int32_t *colidx,
                             const double *H, int64_t F, double *M)
{
    for (int64_t v = 0; v < n_dst; ++v) {
        const double c = 1.0 / ((double)(rowptr[v + 1] - rowptr[v]) + 1.0);
        double *m = M + v * F;
        for (int64_t f = 0; f < F; ++f) m[f] = H[v * F + f];
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            const double *h = H + (int64_t)colidx[e] * F;
            for (int64_t f = 0; f < F; ++f) m[f] += h[f];
        }
        for (int64_t f = 0; f < F; ++f) m[f] *= c;
    }
}

/* out [n_src, F] = (Dt^-1 (A_S + I))^T G, G [n_dst, F]: a scatter over the block. */
void orc_gcn_block_aggregate_T(int64_t n_dst, int64_t n_src, const int32_t *rowptr, const int32_t *colidx,
                               const double *G, int64_t F, double *out)
{
    memset(out, 0, (size_t)(n_src * F) * sizeof(double));
    for (int64_t v = 0; v < n_dst; ++v) {
        const double c = 1.0 / ((double)(rowptr[v + 1] - rowptr[v]) + 1.0);
        for (int64_t f = 0; f < F; ++f) out[v * F + f] += c * G[v * F + f];
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            double *o = out + (int64_t)colidx[e] * F;
            for (int64_t f = 0; f < F; ++f) o[f] += c * G[v * F + f];
        }
    }
}

void orc_gcn_block_layer_fwd(int64_t n_dst, const int32_t *rowptr, const int32_t *colidx,
                             const double *H, int64_t F_in, const double *W, const double *bias,
                             int64_t F_out, int act, double *M, double *Z, double *Hnext)
{
    orc_gcn_block_aggregate(n_dst, rowptr, colidx, H, F_in, M);
    orc_dense_fwd(n_dst, M, F_in, W, bias, F_out, act, Z, Hnext);
}

/* dW = M^T dZ, db = 1^T dZ, dH [n_src, F_in] = (Dt^-1 (A_S + I))^T (dZ W^T)   (dH skipped when NULL).
 * scratch_dM: n_dst*F_in doubles, scratch_dZ: n_dst*F_out doubles. */
void orc_gcn_block_layer_bwd(int64_t n_dst, int64_t n_src, const int32_t *rowptr, const int32_t *colidx,
                             const double *M, const double *Z, const double *dHnext, const double *W,
                             int64_t F_in, int64_t F_out, int act, double *dW, double *dbias, double *dH,
                             double *scratch_dM, double *scratch_dZ)
{
    orc_dense_bwd(n_dst, M, Z, dHnext, W, F_in, F_out, act, dW, dbias, dH ? scratch_dM : NULL, scratch_dZ);
    if (dH) orc_gcn_block_aggregate_T(n_dst, n_src, rowptr, colidx, scratch_dM, F_in, dH);
}

/* ------------------------------------------------------------------------
 * Link-prediction head (Sec. 4.1, paragraphs on the link prediction decoder
 * and on mini-batch and negative sampling; App., formulation of the MLP
 * decoder).
 *
 * Mini-batch: B positive edges drawn uniformly, with replacement, from the
 * local edge list (the directed CSR entries), and for each positive (u, v) one
 * negative (u, v') whose tail v' is uniform over the local nodes other than v.
 * The paper fixes no generator; this build's written spec, with the SplitMix64
 * stream of the partitioner and c = first_counter + i for sample i:
 *     e  = floor(mix64(seed, 2c)   * nnz   / 2^64),  u = row of entry e, v = colidx[e]
 *     r  = floor(mix64(seed, 2c+1) * (n-1) / 2^64),  v' = r + (r >= v)
 * ---------------------------------------------------------------------- */
static int64_t scaled_draw(uint64_t seed, uint64_t counter, uint64_t range)
{
    unsigned __int128 wide = (unsigned __int128)orc_mix64(seed, counter) * range;
    return (int64_t)(wide >> 64);
}

void orc_edge_batch(int64_t n, const int32_t *rowptr, const int32_t *colidx, uint64_t seed,
                    uint64_t first_counter, int64_t B, int32_t *u, int32_t *v, int32_t *vneg)
{
    const int64_t nnz = rowptr[n];
    for (int64_t i = 0; i < B; ++i) {
        const uint64_t c = first_counter + (uint64_t)i;
        const int64_t e = scaled_draw(seed, 2 * c, (uint64_t)nnz);
        int64_t row = 0;
        while (rowptr[row + 1] <= e) ++row;          /* the row whose range holds e */
        const int64_t r = scaled_draw(seed, 2 * c + 1, (uint64_t)(n - 1));
        u[i] = (int32_t)row;
        v[i] = colidx[e];
        vneg[i] = (int32_t)(r + (r >= v[i] ? 1 : 0));
    }
}

/* Decoder input: e0(u, v) = r_u (.) r_v.  Rows 0..B-1 of E0 are the positive
 * pairs (u_i, v_i), rows B..2B-1 the negative pairs (u_i, v'_i). */
void orc_pair_product_fwd(int64_t B, int64_t F, const double *R, const int32_t *u, const int32_t *v,
                          const int32_t *vneg, double *E0)
{
    for (int64_t i = 0; i < B; ++i)
        for (int64_t f = 0; f < F; ++f) {
            E0[i * F + f] = R[(int64_t)u[i] * F + f] * R[(int64_t)v[i] * F + f];
            E0[(B + i) * F + f] = R[(int64_t)u[i] * F + f] * R[(int64_t)vneg[i] * F + f];
        }
}

/* dR = gradient of the pair products w.r.t. the embeddings: every sample adds
 * dE0 (.) (the other factor) to both of its rows; nodes outside the batch get 0. */
void orc_pair_product_bwd(int64_t n, int64_t B, int64_t F, const double *R, const int32_t *u,
                          const int32_t *v, const int32_t *vneg, const double *dE0, double *dR)
{
    memset(dR, 0, (size_t)(n * F) * sizeof(double));
    for (int64_t i = 0; i < B; ++i)
        for (int64_t f = 0; f < F; ++f) {
            const double gp = dE0[i * F + f], gn = dE0[(B + i) * F + f];
            const double ru = R[(int64_t)u[i] * F + f];
            dR[(int64_t)u[i] * F + f] += gp * R[(int64_t)v[i] * F + f] + gn * R[(int64_t)vneg[i] * F + f];
            dR[(int64_t)v[i] * F + f] += gp * ru;
            dR[(int64_t)vneg[i] * F + f] += gn * ru;
        }
}

/* PReLU with one learnable slope (the decoder's activation): y = z > 0 ? z : a z.
 * Backward: dz = dy * (z > 0 ? 1 : a),  da = sum of dy * z over the entries with z <= 0.
 * open_mask (optional, one byte per entry) replaces the decision z > 0. */
void orc_prelu_fwd(int64_t count, const double *Z, double slope, double *Y)
{
    for (int64_t i = 0; i < count; ++i) Y[i] = Z[i] > 0.0 ? Z[i] : slope * Z[i];
}

void orc_prelu_bwd(int64_t count, const double *Z, const double *dY, double slope,
                   const uint8_t *open_mask, double *dZ, double *dslope)
{
    double da = 0.0;
    for (int64_t i = 0; i < count; ++i) {
        const int open = open_mask ? (open_mask[i] != 0) : (Z[i] > 0.0);
        dZ[i] = open ? dY[i] : slope * dY[i];
        if (!open) da += dY[i] * Z[i];
    }
    *dslope = da;
}

/* Binary cross-entropy on logits, mean over all samples; the first n_pos
 * samples are positives (label 1), the rest negatives (label 0).  The paper
 * names the decoder's output the predicted link probability and no loss; this
 * build reads the last layer's scalar as a logit.
 *     loss = mean( y = 1 ? log(1 + exp(-z)) : log(1 + exp(z)) ),  dz = (sigmoid(z) - y) / count */
double orc_bce_logits(int64_t count, int64_t n_pos, const double *z, double *dz)
{
    double loss = 0.0;
    for (int64_t i = 0; i < count; ++i) {
        const double y = i < n_pos ? 1.0 : 0.0;
        const double t = y > 0.5 ? -z[i] : z[i];                  /* loss_i = log(1 + exp(t)) */
        loss += t > 0.0 ? t + log1p(exp(-t)) : log1p(exp(t));
        if (dz) dz[i] = (1.0 / (1.0 + exp(-z[i])) - y) / (double)count;
    }
    return count > 0 ? loss / (double)count : 0.0;
}

/* ------------------------------------------------------------------------
 * Fan-out neighbour sampling for the message-flow graph of a mini-batch
 * (Sec. 4.1, paragraph on mini-batch and negative sampling: the GraphSAGE
 * sampler of Hamilton et al. 2017 caps the neighbours a node aggregates).
 * A node with at most `fanout` local neighbours keeps them all; otherwise a
 * uniformly random subset of exactly `fanout` distinct neighbours is kept.
 * The paper fixes neither sizes nor generator; this build's written spec:
 * entry e of the local CSR gets the key z(e) = mix64(seed, e); a row keeps the
 * `fanout` entries with the smallest (key, e), listed in CSR order.  (Keys are
 * i.i.d., so the kept set is a uniform subset; `seed` is the caller's per step
 * and per layer.)
 *   dst [n_dst]: the local nodes to sample for; blk_rowptr [n_dst+1];
 *   blk_col: kept neighbours (local ids), at most n_dst * fanout.
 * ---------------------------------------------------------------------- */
void orc_neighbor_sample(int64_t n_dst, const int32_t *dst, const int32_t *rowptr, const int32_t *colidx,
                         int32_t fanout, uint64_t seed, int32_t *blk_rowptr, int32_t *blk_col)
{
    int32_t out = 0;
    blk_rowptr[0] = 0;
    for (int64_t i = 0; i < n_dst; ++i) {
        const int32_t beg = rowptr[dst[i]], end = rowptr[dst[i] + 1];
        for (int32_t e = beg; e < end; ++e) {
            int keep = 1;
            if (end - beg > fanout) {          /* rank of (key, e) among the row's entries */
                const uint64_t ke = orc_mix64(seed, (uint64_t)e);
                int32_t smaller = 0;
                for (int32_t o = beg; o < end; ++o) {
                    const uint64_t ko = orc_mix64(seed, (uint64_t)o);
                    if (ko < ke || (ko == ke && o < e)) ++smaller;
                }
                keep = smaller < fanout;
            }
            if (keep) blk_col[out++] = colidx[e];
        }
        blk_rowptr[i + 1] = out;
    }
}
