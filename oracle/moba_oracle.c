/*
 * CPU oracle for Mixture of Block Attention (MoBA), forward and backward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU path and is
 * never called by it; only tests, the smoke check and the benchmark's CPU
 * baseline leg may load it.
 *
 * What it follows (paper: "Optimizing Mixture of Block Attention"):
 *   - Section 2 (Preliminaries): keys are cut into n = N/B blocks; a block's
 *     gate score for a query is the dot product of the query with the block's
 *     mean key (centroid); the k best *past* blocks are kept; the query also
 *     always attends its own block under a causal mask; the output is
 *     softmax(q K_S^T / sqrt(d)) V_S over the selected tokens S.
 *   - Appendix B (Key Convolution Design): k'_t = k_t + SiLU(sum_l W_l * k_{t-l}),
 *     depthwise, causal (terms with t-l < 0 are dropped), applied before the
 *     centroids and before attention; its backward (gradient of K' to K and to the
 *     kernel weights) is the chain rule through that formula.
 *   - Appendix C.3 (backward): D = rowsum(dO o O), P = exp(S - L),
 *     dV = P^T dO, dP = dO V^T, dS = P o (dP - D), dQ = dS K, dK = dS^T Q,
 *     with the 1/sqrt(d) factor of Section 2 restored on S, dQ and dK.
 *
 * Readings taken where the paper is silent (listed again in the design notes):
 *   - top-k counts past blocks only; the own block is extra and never a candidate;
 *   - a query with fewer than k past blocks keeps all of them, the rest is -1;
 *   - equal scores: the lower block index wins;
 *   - gate scores are not scaled by 1/sqrt(d);
 *   - routing is an input of attention and is not differentiated;
 *   - lse is the natural log of the sum of exp of the scaled logits;
 *   - the convolved key is rounded once to the I/O type and that rounded tensor
 *     feeds both the centroids and attention; centroids are stored as fp32;
 *   - in the convolution's backward that rounding is the identity, and the weight
 *     gradient is summed over the batch (the weights are per head and channel).
 *
 * All arithmetic is binary64.  Tensors are row-major [bh, N, d] with
 * bh = batch*heads flattened (head index = slice % heads).
 *
 * parity pins: every function here is pinned by tests/test_oracle_*.py
 * (brute force with an explicit N x N mask, textbook causal attention,
 * closed forms, finite differences, autograd on the dense formulation).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------- rounding helpers ------------------------------------------------ */

/* Round a double to the nearest bfloat16 (ties to even), returned as double.
 * bfloat16 = 1 sign, 8 exponent, 7 fraction bits: 8 significant bits, the
 * smallest normal is 2^-126 and subnormals are multiples of 2^-133. */
static double round_bf16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);            /* |x| = m * 2^e, m in [0.5, 1) */
    int q = e - 8;                 /* exponent of the last kept bit */
    if (q < -133) q = -133;
    return ldexp(rint(ldexp(x, -q)), q);   /* rint: ties-to-even in the default mode */
}

static double round_f32(double x) { return (double)(float)x; }

/* mode 0: fp32, 1: bf16, 2: keep binary64 */
static double round_io(double x, int mode)
{
    return mode == 0 ? round_f32(x) : mode == 1 ? round_bf16(x) : x;
}

void oracle_round_array(const double *in, double *out, int64_t count, int mode)
{
    for (int64_t i = 0; i < count; ++i) out[i] = round_io(in[i], mode);
}

/* ---------- Appendix B: key convolution ------------------------------------ */

/* K, Kp: [bh, N, d];  w: [heads, d, W] with w[h][c][l] the weight of lag l.
 * Kp[t][c] = round_io( K[t][c] + SiLU( sum_{l<W, t-l>=0} w[h][c][l] * K[t-l][c] ) ). */
void oracle_key_conv(const double *K, const double *w, double *Kp,
                     int bh, int heads, int N, int d, int W, int round_mode)
{
    #pragma omp parallel for schedule(static)
    for (int s = 0; s < bh; ++s) {
        const double *Ks = K + (int64_t)s * N * d;
        double *Ps = Kp + (int64_t)s * N * d;
        const double *ws = w + (int64_t)(s % heads) * d * W;
        for (int t = 0; t < N; ++t)
            for (int c = 0; c < d; ++c) {
                double a = 0.0;
                for (int l = 0; l < W; ++l)
                    if (t - l >= 0) a += ws[c * W + l] * Ks[(int64_t)(t - l) * d + c];
                double silu = a / (1.0 + exp(-a));
                Ps[(int64_t)t * d + c] = round_io(Ks[(int64_t)t * d + c] + silu, round_mode);
            }
    }
}

/* Backward of the key convolution (Appendix B: the gradients of the attention go back through
 * the convolution to the token-level keys and to the kernel weights).  With
 * a[t][c] = sum_{l<W, t-l>=0} w[h][c][l] K[t-l][c] and K' = K + SiLU(a) (the rounding of K' to
 * the storage type is treated as the identity), G = dL/dK':
 *   g[t][c]   = G[t][c] * SiLU'(a[t][c]),   SiLU'(x) = s(x) (1 + x (1 - s(x))),  s = sigmoid
 *   dK[t][c]  = G[t][c] + sum_{l<W, t+l<N} w[h][c][l] g[t+l][c]
 *   dw[h][c][l] = sum over the slices of head h and over t >= l of  g[t][c] K[t-l][c]
 * K, G, dK: [bh, N, d];  w, dw: [heads, d, W] (the weights are shared across the batch). */
void oracle_key_conv_bwd(const double *K, const double *w, const double *G, double *dK, double *dw,
                         int bh, int heads, int N, int d, int W)
{
    for (int64_t i = 0; i < (int64_t)heads * d * W; ++i) dw[i] = 0.0;
    double *g = (double *)malloc(sizeof(double) * (size_t)N * d);
    for (int s = 0; s < bh; ++s) {
        const double *Ks = K + (int64_t)s * N * d, *Gs = G + (int64_t)s * N * d;
        double *dKs = dK + (int64_t)s * N * d;
        const double *ws = w + (int64_t)(s % heads) * d * W;
        double *dws = dw + (int64_t)(s % heads) * d * W;
        for (int t = 0; t < N; ++t)
            for (int c = 0; c < d; ++c) {
                double a = 0.0;
                for (int l = 0; l < W; ++l)
                    if (t - l >= 0) a += ws[c * W + l] * Ks[(int64_t)(t - l) * d + c];
                double sg = 1.0 / (1.0 + exp(-a));
                g[(int64_t)t * d + c] = Gs[(int64_t)t * d + c] * sg * (1.0 + a * (1.0 - sg));
            }
        for (int t = 0; t < N; ++t)
            for (int c = 0; c < d; ++c) {
                double acc = Gs[(int64_t)t * d + c];
                for (int l = 0; l < W; ++l)
                    if (t + l < N) acc += ws[c * W + l] * g[(int64_t)(t + l) * d + c];
                dKs[(int64_t)t * d + c] = acc;
            }
        for (int c = 0; c < d; ++c)
            for (int l = 0; l < W; ++l) {
                double acc = 0.0;
                for (int t = l; t < N; ++t) acc += g[(int64_t)t * d + c] * Ks[(int64_t)(t - l) * d + c];
                dws[c * W + l] += acc;
            }
    }
    free(g);
}

/* ---------- Section 2: centroids -------------------------------------------- */

/* C[s][j][:] = mean of the B keys of block j, rounded to fp32 (the stored type). */
void oracle_centroids(const double *K, double *C, int bh, int N, int d, int B)
{
    int n = N / B;
    #pragma omp parallel for schedule(static)
    for (int64_t sj = 0; sj < (int64_t)bh * n; ++sj) {
        const double *Kb = K + sj * B * d;     /* block j of slice s starts at row j*B */
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int r = 0; r < B; ++r) acc += Kb[(int64_t)r * d + c];
            C[sj * d + c] = round_f32(acc / (double)B);
        }
    }
}

/* ---------- Section 2: gate scores and causal top-k ------------------------- */

/* Gate scores of a list of query rows against every block (future and own
 * blocks get -inf).  rows[i] = s*N + t.  S: [nrows, n]. */
void oracle_gate_scores(const double *Q, const double *C, const int64_t *rows, int64_t nrows,
                        double *S, int N, int d, int B)
{
    int n = N / B;
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t s = rows[i] / N; int t = (int)(rows[i] % N);
        int own = t / B;
        const double *q = Q + rows[i] * d;
        for (int j = 0; j < n; ++j) {
            if (j >= own) { S[i * n + j] = -INFINITY; continue; }
            const double *c = C + ((int64_t)s * n + j) * d;
            double acc = 0.0;
            for (int x = 0; x < d; ++x) acc += q[x] * c[x];
            S[i * n + j] = acc;
        }
    }
}

/* Top-k of a list of query rows.  rows[i] = s*N + t.
 * idx: [nrows, k] int32, best first, -1 in unused slots.
 * kth: [nrows] score of the last selected block (NaN when none is selected). */
void oracle_topk(const double *Q, const double *C, const int64_t *rows, int64_t nrows,
                 int32_t *idx, double *kth, int N, int d, int B, int k)
{
    int n = N / B;
    #pragma omp parallel
    {
        double *sc = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        char *taken = (char *)malloc((size_t)(n > 0 ? n : 1));
        #pragma omp for schedule(dynamic, 64)
        for (int64_t i = 0; i < nrows; ++i) {
            int64_t r = rows[i], s = r / N; int t = (int)(r % N);
            int past = t / B;                      /* blocks 0..past-1 are candidates */
            const double *q = Q + r * d;
            for (int j = 0; j < past; ++j) {
                const double *c = C + ((int64_t)s * n + j) * d;
                double acc = 0.0;
                for (int x = 0; x < d; ++x) acc += q[x] * c[x];
                sc[j] = acc; taken[j] = 0;
            }
            int keep = past < k ? past : k;
            double last = NAN;
            for (int slot = 0; slot < k; ++slot) {
                if (slot >= keep) { idx[i * k + slot] = -1; continue; }
                int best = -1;
                for (int j = 0; j < past; ++j)        /* strict > keeps the lower index on ties */
                    if (!taken[j] && (best < 0 || sc[j] > sc[best])) best = j;
                taken[best] = 1;
                idx[i * k + slot] = best;
                last = sc[best];
            }
            kth[i] = last;
        }
        free(sc); free(taken);
    }
}

/* ---------- Appendix C.1: key-block-major query lists ------------------------ */

/* off: [bh, n+1] exclusive prefix sums of the per-block counts;
 * qlist: [bh, R] query ids, ascending inside each block's segment, where R is the
 * number of (query, selected past block) pairs of one slice (the same for every slice).
 * Returns R, or -1 if slices disagree. */
int64_t oracle_csr(const int32_t *idx, int32_t *off, int32_t *qlist,
                   int bh, int N, int B, int k, int64_t R)
{
    int n = N / B;
    for (int s = 0; s < bh; ++s) {
        int32_t *o = off + (int64_t)s * (n + 1);
        memset(o, 0, sizeof(int32_t) * (size_t)(n + 1));
        const int32_t *is = idx + (int64_t)s * N * k;
        for (int64_t e = 0; e < (int64_t)N * k; ++e)
            if (is[e] >= 0) o[is[e] + 1]++;
        for (int j = 0; j < n; ++j) o[j + 1] += o[j];
        if (o[n] != R) return -1;
        int32_t *fill = (int32_t *)calloc((size_t)(n > 0 ? n : 1), sizeof(int32_t));
        int32_t *ql = qlist + (int64_t)s * R;
        for (int t = 0; t < N; ++t)                  /* ascending t gives ascending lists */
            for (int c = 0; c < k; ++c) {
                int32_t b = is[(int64_t)t * k + c];
                if (b >= 0) ql[o[b] + fill[b]++] = t;
            }
        free(fill);
    }
    return R;
}

/* ---------- Section 2: attention over the selected tokens ------------------- */

/* One query row.  z_u = scale * q.k_u over u in the selected past blocks and
 * over u <= t in the own block; softmax; O = sum P_u v_u; lse = m + log sum e^{z-m}.
 * p_out (optional) receives the logits z in visiting order, for reuse. */
static void attend_row(const double *Qs, const double *Ks, const double *Vs, const int32_t *sel,
                       int t, int d, int B, int k, double scale, double *O, double *lse,
                       double *zbuf)
{
    const double *q = Qs + (int64_t)t * d;
    int own = t / B, cnt = 0;
    double m = -INFINITY;
    for (int c = 0; c <= k; ++c) {
        int blk = (c < k) ? sel[c] : own;
        if (blk < 0) continue;
        int hi = (c < k) ? (blk + 1) * B - 1 : t;      /* own block: keys up to t only */
        for (int u = blk * B; u <= hi; ++u) {
            const double *ku = Ks + (int64_t)u * d;
            double acc = 0.0;
            for (int x = 0; x < d; ++x) acc += q[x] * ku[x];
            double z = scale * acc;
            zbuf[cnt++] = z;
            if (z > m) m = z;
        }
    }
    double l = 0.0;
    for (int i = 0; i < cnt; ++i) l += exp(zbuf[i] - m);
    for (int x = 0; x < d; ++x) O[x] = 0.0;
    cnt = 0;
    for (int c = 0; c <= k; ++c) {
        int blk = (c < k) ? sel[c] : own;
        if (blk < 0) continue;
        int hi = (c < k) ? (blk + 1) * B - 1 : t;
        for (int u = blk * B; u <= hi; ++u) {
            double p = exp(zbuf[cnt++] - m) / l;
            const double *vu = Vs + (int64_t)u * d;
            for (int x = 0; x < d; ++x) O[x] += p * vu[x];
        }
    }
    *lse = m + log(l);
}

/* rows[i] = s*N + t.  O: [nrows, d], lse: [nrows]. */
void oracle_attn_fwd(const double *Q, const double *K, const double *V, const int32_t *idx,
                     const int64_t *rows, int64_t nrows, double *O, double *lse,
                     int N, int d, int B, int k, double scale)
{
    #pragma omp parallel
    {
        double *zbuf = (double *)malloc(sizeof(double) * (size_t)(k + 1) * B);
        #pragma omp for schedule(dynamic, 16)
        for (int64_t i = 0; i < nrows; ++i) {
            int64_t s = rows[i] / N; int t = (int)(rows[i] % N);
            attend_row(Q + s * N * d, K + s * N * d, V + s * N * d, idx + rows[i] * k,
                       t, d, B, k, scale, O + i * d, lse + i, zbuf);
        }
        free(zbuf);
    }
}

/* ---------- Appendix C.3: backward with the routing held fixed --------------- */

/* dQ of a list of query rows.  lse and Dv are full [bh, N] arrays (only the
 * listed rows are read): lse from the forward, Dv[t] = dO_t . O_t.
 * dQ_t = scale * sum_u dS_tu k_u,  dS_tu = P_tu (dO_t.v_u - D_t),  P_tu = exp(z_tu - lse_t). */
void oracle_attn_bwd_dq(const double *Q, const double *K, const double *V, const int32_t *idx,
                        const double *dO, const double *lse, const double *Dv,
                        const int64_t *rows, int64_t nrows, double *dQ,
                        int N, int d, int B, int k, double scale)
{
    #pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t r = rows[i], s = r / N; int t = (int)(r % N);
        const double *q = Q + r * d, *g = dO + r * d;
        const double *Ks = K + s * N * d, *Vs = V + s * N * d;
        const int32_t *sel = idx + r * k;
        double *out = dQ + i * d;
        for (int x = 0; x < d; ++x) out[x] = 0.0;
        int own = t / B;
        for (int c = 0; c <= k; ++c) {
            int blk = (c < k) ? sel[c] : own;
            if (blk < 0) continue;
            int hi = (c < k) ? (blk + 1) * B - 1 : t;
            for (int u = blk * B; u <= hi; ++u) {
                const double *ku = Ks + (int64_t)u * d, *vu = Vs + (int64_t)u * d;
                double z = 0.0, dp = 0.0;
                for (int x = 0; x < d; ++x) { z += q[x] * ku[x]; dp += g[x] * vu[x]; }
                double p = exp(scale * z - lse[r]);
                double ds = p * (dp - Dv[r]);
                for (int x = 0; x < d; ++x) out[x] += scale * ds * ku[x];
            }
        }
    }
}

/* dK, dV of a list of key blocks.  blocks[i] = s*n + j.  off/qlist are the
 * key-block-major lists of the routing (oracle_csr).  The queries that see block j
 * are the listed ones (every key of the block) and the block's own queries
 * (keys u <= t).  dK, dV: [nblocks, B, d].
 * dV_u = sum_t P_tu dO_t,  dK_u = scale * sum_t dS_tu q_t. */
void oracle_attn_bwd_dkdv(const double *Q, const double *K, const double *V,
                          const double *dO, const double *lse, const double *Dv,
                          const int32_t *off, const int32_t *qlist, int64_t R,
                          const int64_t *blocks, int64_t nblocks, double *dK, double *dV,
                          int N, int d, int B, double scale)
{
    int n = N / B;
    #pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < nblocks; ++i) {
        int64_t s = blocks[i] / n; int j = (int)(blocks[i] % n);
        const int32_t *o = off + s * (n + 1);
        const int32_t *ql = qlist + s * R;
        int nlist = o[j + 1] - o[j];
        double *dKb = dK + i * B * d, *dVb = dV + i * B * d;
        for (int64_t e = 0; e < (int64_t)B * d; ++e) dKb[e] = dVb[e] = 0.0;
        for (int a = 0; a < nlist + B; ++a) {
            int t = (a < nlist) ? ql[o[j] + a] : j * B + (a - nlist);
            int hi = (a < nlist) ? (j + 1) * B - 1 : t;
            int64_t r = s * N + t;
            const double *q = Q + r * d, *g = dO + r * d;
            for (int u = j * B; u <= hi; ++u) {
                const double *ku = K + (s * N + u) * d, *vu = V + (s * N + u) * d;
                double z = 0.0, dp = 0.0;
                for (int x = 0; x < d; ++x) { z += q[x] * ku[x]; dp += g[x] * vu[x]; }
                double p = exp(scale * z - lse[r]);
                double ds = p * (dp - Dv[r]);
                double *dk = dKb + (int64_t)(u - j * B) * d, *dv = dVb + (int64_t)(u - j * B) * d;
                for (int x = 0; x < d; ++x) { dv[x] += p * g[x]; dk[x] += scale * ds * q[x]; }
            }
        }
    }
}

int oracle_num_threads(void)
{
    int nt = 1;
    #pragma omp parallel
    {
        #pragma omp master
        {
#ifdef _OPENMP
            extern int omp_get_num_threads(void);
            nt = omp_get_num_threads();
#endif
        }
    }
    return nt;
}
