/*
 * vfa_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, float64 CPU implementation of what the VFA / VSA attention
 * forward path computes.  It exists so that the GPU library can be checked
 * against something written directly from the paper.  It shares no code,
 * header, table or helper with the GPU library, and the GPU library never
 * calls it.  Only tests, the smoke check and the benchmark's cpu_baseline
 * leg may load it.
 *
 * What each function follows:
 *   oracle_brute      Sec. 2.1: S = Q K^T / sqrt(d), P = softmax(S), O = P V, with
 *                     the whole N x N matrix materialised (tiny inputs only).
 *   oracle_exact      the same definition, row by row in two passes (max, then
 *                     sum), for chosen query blocks of a large problem.
 *   oracle_sabsmax    Alg. 1, its first loop (one summary per key block), and the
 *                     sentence defining sabsmax in Methods, Step 1.
 *   oracle_visit_list Alg. 1 main-loop order <1, i, 2, 3, ...> (Step 2),
 *                     generalised as stated below.
 *   oracle_blocks     Alg. 1 (VFA), Alg. 2 (VSA) and the FA column of Table 1
 *                     (online softmax on every block), selected by switches.
 *   oracle_e4m3_* / oracle_mx_*  the published FP8 and MX (E2M1 / E5M2 with shared E8M0 scales)
 *                     codecs for the low-precision tensor regimes of the performance
 *                     discussion; the attention itself is then checked on the
 *                     dequantised operands with the functions above.
 *
 * Readings taken where the paper is silent or inconsistent (all 0-based here;
 * the paper counts blocks from 1):
 *   R1  The 1/sqrt(d) scale of Sec. 2.1 / Table 1 "MUL" applies to S and to the
 *       approximate scores alike (Alg. 1 omits it in both).
 *   R2  sabsmax tie (+a and -a both of largest magnitude): the positive one.
 *   R3  One summary per main-loop key block (T_c1 = T_c, as the paper sets it).
 *   R4  Causal: m-init runs over visible key blocks only (j <= j_hi(i)).
 *   R5  Special set = the first n_sink blocks, and the local set L(i) = the key
 *       blocks overlapping the query block's own token range, plus the
 *       n_local-1 blocks just before them; each block is visited once; order
 *       inside each group ascending.  With block_m == block_n and
 *       n_sink = n_local = 1 this is the paper's {1, i}.
 *   R6  Causal masking: S = -inf where key index > query index; a fully masked
 *       row keeps its state.
 *   R7  VSA: a block is skipped iff the skip inequality holds for ALL rows of
 *       the query block (rows with no visible key in the block vote "skip").
 *       PARITY UNPINNED: the paper prints no value that fixes this reading;
 *       it is supported only by the row-skip variant's description.
 *   R8  VSA: the test uses m* = max(m_prev, m~); a skipped block leaves the
 *       state unchanged, also when it is a special block.
 *   R9  All blocks of a row skipped => l = 0 => O = 0, LSE = -inf.
 *   R10 LSE = m + ln(l) (natural log, scaled scores).  The paper outputs only
 *       O; PARITY UNPINNED by the paper, pinned here by the brute-force
 *       definition ln(sum exp(s)).
 *
 * All tensors are row-major: Q [B,Hq,N,d], K,V [B,Hkv,N,d] as float32 on input
 * (bf16-representable values widen exactly), everything inside is double.
 * Query head h reads KV head h / (Hq/Hkv).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    const float *Q, *K, *V;
    int B, Hq, Hkv, N, d;
    int block_m, block_n;
    int causal;
    double scale;
} prob_t;

static int ceil_div(int a, int b) { return (a + b - 1) / b; }
static int imin(int a, int b) { return a < b ? a : b; }
static int imax(int a, int b) { return a > b ? a : b; }

static const float *q_row(const prob_t *p, int b, int h, int r) {
    return p->Q + (((size_t)b * p->Hq + h) * p->N + r) * p->d;
}
static const float *k_row(const prob_t *p, int b, int h, int c) {
    int hkv = h / (p->Hq / p->Hkv);
    return p->K + (((size_t)b * p->Hkv + hkv) * p->N + c) * p->d;
}
static const float *v_row(const prob_t *p, int b, int h, int c) {
    int hkv = h / (p->Hq / p->Hkv);
    return p->V + (((size_t)b * p->Hkv + hkv) * p->N + c) * p->d;
}

/* s = scale * <Q[r], K[c]>   (Sec. 2.1) */
static double score(const prob_t *p, int b, int h, int r, int c) {
    const float *q = q_row(p, b, h, r), *k = k_row(p, b, h, c);
    double acc = 0.0;
    for (int t = 0; t < p->d; ++t) acc += (double)q[t] * (double)k[t];
    return p->scale * acc;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Brute force, one head: S [N,N], P = softmax rows, O = P V.          */
/* P_out [N,N] and O_out [N,d], LSE_out [N]; Q,K,V are [N,d].           */
int oracle_brute(const float *Q, const float *K, const float *V, int N, int d, int causal,
                 double scale, double *P_out, double *O_out, double *LSE_out) {
    prob_t p = {Q, K, V, 1, 1, 1, N, d, N, N, causal, scale};
    double *S = (double *)malloc((size_t)N * N * sizeof(double));
    if (!S) return -1;
    for (int r = 0; r < N; ++r)
        for (int c = 0; c < N; ++c)
            S[(size_t)r * N + c] = (causal && c > r) ? -INFINITY : score(&p, 0, 0, r, c);
    for (int r = 0; r < N; ++r) {
        double mx = -INFINITY, sum = 0.0;
        for (int c = 0; c < N; ++c) mx = fmax(mx, S[(size_t)r * N + c]);
        for (int c = 0; c < N; ++c) sum += exp(S[(size_t)r * N + c] - mx);
        for (int c = 0; c < N; ++c) P_out[(size_t)r * N + c] = exp(S[(size_t)r * N + c] - mx) / sum;
        LSE_out[r] = mx + log(sum);
        for (int t = 0; t < d; ++t) {
            double acc = 0.0;
            for (int c = 0; c < N; ++c) acc += P_out[(size_t)r * N + c] * (double)V[(size_t)c * d + t];
            O_out[(size_t)r * d + t] = acc;
        }
    }
    free(S);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Exact attention for listed query blocks.  blocks = nblk triples (b, h, i).
 * O [nblk, block_m, d], LSE [nblk, block_m], M [nblk, block_m] (true row max).
 * Rows beyond N are left untouched.                                     */
int oracle_exact(const float *Q, const float *K, const float *V, int B, int Hq, int Hkv, int N,
                 int d, int block_m, int causal, double scale, int nblk, const int *blocks,
                 double *O, double *LSE, double *M) {
    prob_t p = {Q, K, V, B, Hq, Hkv, N, d, block_m, block_m, causal, scale};
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < nblk; ++n) {
        int b = blocks[3 * n], h = blocks[3 * n + 1], i = blocks[3 * n + 2];
        double *s = (double *)malloc((size_t)N * sizeof(double));
        for (int rr = 0; rr < block_m; ++rr) {
            int r = i * block_m + rr;
            if (r >= N) break;
            int nvis = causal ? r + 1 : N;
            double mx = -INFINITY, sum = 0.0;
            for (int c = 0; c < nvis; ++c) { s[c] = score(&p, b, h, r, c); mx = fmax(mx, s[c]); }
            for (int c = 0; c < nvis; ++c) { s[c] = exp(s[c] - mx); sum += s[c]; }
            double *o = O + ((size_t)n * block_m + rr) * d;
            for (int t = 0; t < d; ++t) o[t] = 0.0;
            for (int c = 0; c < nvis; ++c) {
                const float *v = v_row(&p, b, h, c);
                for (int t = 0; t < d; ++t) o[t] += s[c] * (double)v[t];
            }
            for (int t = 0; t < d; ++t) o[t] /= sum;
            LSE[(size_t)n * block_m + rr] = mx + log(sum);
            M[(size_t)n * block_m + rr] = mx;
        }
        free(s);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* sabsmax (Alg. 1 precompute; Step 1): per key block and dimension, the
 * element of largest absolute value with its sign; reading R2 on ties.
 * repr_mode: 0 sabsmax (the method); 1 per-dim max; 2 per-dim mean;
 * 3 unsigned absmax (the three ablated summaries).  out [B,Hkv,Tc,d].    */
int oracle_sabsmax(const float *K, int B, int Hkv, int N, int d, int block_n, int repr_mode,
                   double *out) {
    int Tc = ceil_div(N, block_n);
    for (int bh = 0; bh < B * Hkv; ++bh)
        for (int j = 0; j < Tc; ++j)
            for (int t = 0; t < d; ++t) {
                int c0 = j * block_n, c1 = imin(N, c0 + block_n);
                double best = (double)K[((size_t)bh * N + c0) * d + t];
                double sum = 0.0, mx = -INFINITY, amx = 0.0;
                for (int c = c0; c < c1; ++c) {
                    double x = (double)K[((size_t)bh * N + c) * d + t];
                    if (fabs(x) > fabs(best) || (fabs(x) == fabs(best) && x > best)) best = x;
                    sum += x;
                    mx = fmax(mx, x);
                    amx = fmax(amx, fabs(x));
                }
                double r = best;
                if (repr_mode == 1) r = mx;
                if (repr_mode == 2) r = sum / (c1 - c0);
                if (repr_mode == 3) r = amx;
                out[((size_t)bh * Tc + j) * d + t] = r;
            }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Block geometry (reading R5).  a_lo..a_hi: key blocks overlapping the
 * query block's own tokens; j_hi: last visible key block.              */
static void geometry(int N, int block_m, int block_n, int causal, int i, int *a_lo, int *a_hi,
                     int *j_hi) {
    int r0 = i * block_m, r1 = imin(N, r0 + block_m) - 1;
    *a_lo = r0 / block_n;
    *a_hi = r1 / block_n;
    *j_hi = causal ? *a_hi : ceil_div(N, block_n) - 1;
}

/* Visit order of Alg. 1's main loop for query block i.
 * reorder = 1: sink blocks, then local blocks, then the rest, each once.
 * reorder = 0: plain ascending order ("w/o reorder" ablation, and FA).
 * special_out[k] = 1 where the block takes the exact-max update.
 * Returns the number of visited blocks; arrays must hold Tc entries.    */
int oracle_visit_list(int N, int block_m, int block_n, int causal, int i, int n_sink, int n_local,
                      int reorder, int *j_out, int *special_out) {
    int a_lo, a_hi, j_hi;
    geometry(N, block_m, block_n, causal, i, &a_lo, &a_hi, &j_hi);
    int Tc = ceil_div(N, block_n);
    char *is_special = (char *)calloc((size_t)Tc, 1), *seen = (char *)calloc((size_t)Tc, 1);
    for (int j = 0; j < n_sink && j <= j_hi; ++j) is_special[j] = 1;
    if (n_local > 0)
        for (int j = imax(0, a_lo - (n_local - 1)); j <= imin(a_hi, j_hi); ++j) is_special[j] = 1;
    int n = 0;
    if (reorder) {
        for (int j = 0; j < n_sink && j <= j_hi; ++j)
            if (!seen[j]) { seen[j] = 1; j_out[n] = j; special_out[n++] = 1; }
        if (n_local > 0)
            for (int j = imax(0, a_lo - (n_local - 1)); j <= imin(a_hi, j_hi); ++j)
                if (!seen[j]) { seen[j] = 1; j_out[n] = j; special_out[n++] = 1; }
    }
    for (int j = 0; j <= j_hi; ++j)
        if (!seen[j]) { seen[j] = 1; j_out[n] = j; special_out[n++] = is_special[j]; }
    free(is_special);
    free(seen);
    return n;
}

/* ------------------------------------------------------------------ */
/* One query block of Alg. 1 / Alg. 2 / FA.  See oracle_blocks for the
 * meaning of the switches and outputs.                                  */
typedef struct {
    int n_sink, n_local, use_minit, reorder, freeze, vsa;
    double ln_lambda;
    const double *qrepr; /* NULL, or [B,Hq,Tr,d]: one summary vector per query block replaces the rows of
                          * Q_i in the approximate score (the ablation that approximates block-wise on Q) */
} opts_t;

/* One query block of Alg. 1 (VFA), Alg. 2 (VSA: vsa = 1) or the FA column of Table 1 (freeze = 0,
 * ascending order, no seed), in the algorithms' order of steps.  The appendix variants with their
 * extra rules live in one_block_variant below. */

static void one_block(const prob_t *p, const opts_t *o, const double *krepr, int b, int h, int i,
                      const double *m_override, double *O, double *LSE, double *m_init_out,
                      double *m_final_out, uint8_t *mask_row, double *margin_row,
                      int64_t *counters, double *traj) {
    const int N = p->N, d = p->d, Br = p->block_m, Bc = p->block_n;
    const int Tc = ceil_div(N, Bc);
    const int r0 = i * Br, nr = imin(Br, N - r0);
    const int hkv = h / (p->Hq / p->Hkv);
    int a_lo, a_hi, j_hi;
    geometry(N, Br, Bc, p->causal, i, &a_lo, &a_hi, &j_hi);

    double *m = (double *)malloc((size_t)Br * sizeof(double));
    double *l = (double *)calloc((size_t)Br, sizeof(double));
    double *acc = (double *)calloc((size_t)Br * d, sizeof(double));
    double *S = (double *)malloc((size_t)Br * Bc * sizeof(double));
    double *mt = (double *)malloc((size_t)Br * sizeof(double));
    int *vj = (int *)malloc((size_t)Tc * sizeof(int)), *vs = (int *)malloc((size_t)Tc * sizeof(int));

    /* m-initialisation (Alg. 1: score_approx = Q_i k_repr_j^T, elementwise max over j).  In the
     * block-wise ablation the score is q_repr_i k_repr_j^T, one scalar per key block, and every
     * row of the query block starts from the same maximum. */
    for (int rr = 0; rr < nr; ++rr) {
        double mi = -INFINITY;
        if (o->use_minit) {
            const float *q = q_row(p, b, h, r0 + rr);
            const double *qr = o->qrepr
                ? o->qrepr + (((size_t)b * p->Hq + h) * ceil_div(N, Br) + i) * d : NULL;
            for (int j = 0; j <= j_hi; ++j) {
                const double *kr = krepr + (((size_t)b * p->Hkv + hkv) * Tc + j) * d;
                double a = 0.0;
                for (int t = 0; t < d; ++t) a += (qr ? qr[t] : (double)q[t]) * kr[t];
                mi = fmax(mi, p->scale * a);
            }
        }
        if (m_override) mi = m_override[rr];
        m[rr] = mi;
        if (m_init_out) m_init_out[rr] = mi;
    }
    if (mask_row) for (int j = 0; j < Tc; ++j) mask_row[j] = 2; /* not visited */
    if (margin_row) for (int j = 0; j < Tc; ++j) margin_row[j] = NAN;

    int nv = oracle_visit_list(N, Br, Bc, p->causal, i, o->n_sink, o->n_local, o->reorder, vj, vs);
    for (int k = 0; k < nv; ++k) {
        const int j = vj[k];
        const int special = o->freeze ? vs[k] : 1;
        const int c0 = j * Bc, nc = imin(Bc, N - c0);
        /* S_ij = scale * Q_i K_j^T, masked entries -inf */
        for (int rr = 0; rr < nr; ++rr)
            for (int cc = 0; cc < nc; ++cc) {
                int r = r0 + rr, c = c0 + cc;
                S[rr * Bc + cc] = (p->causal && c > r) ? -INFINITY : score(p, b, h, r, c);
            }
        counters[0] += 1; /* visited tiles */
        if (o->vsa || special) {
            for (int rr = 0; rr < nr; ++rr) {
                double x = -INFINITY;
                for (int cc = 0; cc < nc; ++cc) x = fmax(x, S[rr * Bc + cc]);
                mt[rr] = x;
            }
            counters[1] += 1; /* rowmax executed on this tile */
        }
        if (o->vsa) {
            /* Alg. 2: m* = max(m_prev, m~); skip iff m~ - m* < ln(lambda) for all rows */
            double worst = -INFINITY;
            for (int rr = 0; rr < nr; ++rr) {
                double diff;
                if (mt[rr] == -INFINITY) diff = -INFINITY;
                else diff = mt[rr] - fmax(m[rr], mt[rr]);
                worst = fmax(worst, diff);
            }
            if (margin_row) margin_row[j] = worst - o->ln_lambda;
            if (worst < o->ln_lambda) {
                if (mask_row) mask_row[j] = 1;
                counters[3] += 1; /* skipped tiles */
                if (traj) for (int rr = 0; rr < nr; ++rr) { traj[((size_t)k * Br + rr) * 2] = m[rr]; traj[((size_t)k * Br + rr) * 2 + 1] = l[rr]; }
                continue;
            }
        }
        if (mask_row) mask_row[j] = 0;
        if (special) counters[2] += 1; /* rescale chain executed on this tile */
        for (int rr = 0; rr < nr; ++rr) {
            double m_use = m[rr], alpha = 1.0;
            if (special) {
                double m_new = fmax(m[rr], mt[rr]);
                alpha = (m_new == -INFINITY) ? 1.0 : exp(m[rr] - m_new);
                m_use = m_new;
            }
            double rowsum = 0.0;
            double *orow = acc + (size_t)rr * d;
            if (special) {
                for (int t = 0; t < d; ++t) orow[t] *= alpha;
                l[rr] *= alpha;
            }
            for (int cc = 0; cc < nc; ++cc) {
                double s = S[rr * Bc + cc];
                double pt = (s == -INFINITY) ? 0.0 : exp(s - m_use);
                rowsum += pt;
                const float *v = v_row(p, b, h, c0 + cc);
                for (int t = 0; t < d; ++t) orow[t] += pt * (double)v[t];
            }
            l[rr] += rowsum;
            m[rr] = m_use;
        }
        if (traj) for (int rr = 0; rr < nr; ++rr) { traj[((size_t)k * Br + rr) * 2] = m[rr]; traj[((size_t)k * Br + rr) * 2 + 1] = l[rr]; }
    }
    /* final normalisation O = O / l */
    for (int rr = 0; rr < nr; ++rr) {
        for (int t = 0; t < d; ++t) O[(size_t)rr * d + t] = (l[rr] > 0.0) ? acc[(size_t)rr * d + t] / l[rr] : 0.0;
        LSE[rr] = (l[rr] > 0.0) ? m[rr] + log(l[rr]) : -INFINITY;
        if (m_final_out) m_final_out[rr] = m[rr];
    }
    free(m); free(l); free(acc); free(S); free(mt); free(vj); free(vs);
}

/* Listed query blocks of VFA (Alg. 1), VSA (Alg. 2) or FA (Table 1, FA column).
 *
 *   blocks      nblk triples (b, h, i)
 *   krepr       [B,Hkv,Tc,d] from oracle_sabsmax (ignored when use_minit = 0)
 *   n_sink, n_local, use_minit   as in the method (use_minit = 0: m starts at -inf)
 *   reorder     1 = sink, local, rest (the method); 0 = ascending order
 *   freeze      1 = exact-max update on special blocks only (the method);
 *               0 = on every block (FA / online softmax)
 *   vsa         1 = Alg. 2 skip test on every visited block, threshold ln_lambda < 0
 *   m_override  NULL, or [nblk, block_m] values that replace m_init (test hook for
 *               the identity "any finite seed gives the exact result")
 *   O [nblk,block_m,d]  LSE [nblk,block_m]
 *   m_init_out, m_final_out  NULL or [nblk, block_m]
 *   mask_out    NULL or [nblk, Tc] uint8: 0 computed, 1 skipped, 2 not visited
 *   margin_out  NULL or [nblk, Tc]: max_r(m~ - m*) - ln_lambda (skip iff < 0), NaN if not visited
 *   counters    [nblk, 4] int64: tiles visited, rowmax executions, rescale executions, skipped
 *   traj        NULL or [nblk, Tc, block_m, 2]: (m, l) after the k-th visited block
 * FA is (use_minit=0, reorder=0, freeze=0, vsa=0).                       */
int oracle_blocks_qrepr(const float *Q, const float *K, const float *V, int B, int Hq, int Hkv, int N,
                        int d, int block_m, int block_n, int causal, double scale, const double *krepr,
                        const double *qrepr, int n_sink, int n_local, int use_minit, int reorder,
                        int freeze, int vsa, double ln_lambda, int nblk, const int *blocks,
                        const double *m_override, double *O, double *LSE, double *m_init_out,
                        double *m_final_out, uint8_t *mask_out, double *margin_out,
                        int64_t *counters, double *traj);

int oracle_blocks(const float *Q, const float *K, const float *V, int B, int Hq, int Hkv, int N,
                  int d, int block_m, int block_n, int causal, double scale, const double *krepr,
                  int n_sink, int n_local, int use_minit, int reorder, int freeze, int vsa,
                  double ln_lambda, int nblk, const int *blocks, const double *m_override,
                  double *O, double *LSE, double *m_init_out, double *m_final_out,
                  uint8_t *mask_out, double *margin_out, int64_t *counters, double *traj) {
    return oracle_blocks_qrepr(Q, K, V, B, Hq, Hkv, N, d, block_m, block_n, causal, scale, krepr, NULL,
                               n_sink, n_local, use_minit, reorder, freeze, vsa, ln_lambda, nblk,
                               blocks, m_override, O, LSE, m_init_out, m_final_out, mask_out,
                               margin_out, counters, traj);
}

/* oracle_blocks with the left operand of the approximate score ablated (Experiments, "Replacing
 * row-wise approximation with block-wise approximation on Q"): qrepr [B,Hq,ceil(N/block_m),d] holds
 * one summary of each query block (oracle_sabsmax applied to Q with block_m gives the three
 * summaries the ablation table lists); the score q_repr_i . k_repr_j is broadcast to all rows of
 * block i.  qrepr = NULL is the row-wise method. */
int oracle_blocks_qrepr(const float *Q, const float *K, const float *V, int B, int Hq, int Hkv, int N,
                        int d, int block_m, int block_n, int causal, double scale, const double *krepr,
                        const double *qrepr, int n_sink, int n_local, int use_minit, int reorder,
                        int freeze, int vsa, double ln_lambda, int nblk, const int *blocks,
                        const double *m_override, double *O, double *LSE, double *m_init_out,
                        double *m_final_out, uint8_t *mask_out, double *margin_out,
                        int64_t *counters, double *traj) {
    if (Hq % Hkv != 0 || block_m <= 0 || block_n <= 0) return -1;
    if (use_minit && !krepr && !m_override) return -1;
    prob_t p = {Q, K, V, B, Hq, Hkv, N, d, block_m, block_n, causal, scale};
    opts_t o = {n_sink, n_local, use_minit, reorder, freeze, vsa, ln_lambda, qrepr};
    const int Tc = ceil_div(N, block_n);
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < nblk; ++n) {
        int64_t *cn = counters + (size_t)n * 4;
        cn[0] = cn[1] = cn[2] = cn[3] = 0;
        one_block(&p, &o, krepr, blocks[3 * n], blocks[3 * n + 1], blocks[3 * n + 2],
                  m_override ? m_override + (size_t)n * block_m : NULL,
                  O + (size_t)n * block_m * d, LSE + (size_t)n * block_m,
                  m_init_out ? m_init_out + (size_t)n * block_m : NULL,
                  m_final_out ? m_final_out + (size_t)n * block_m : NULL,
                  mask_out ? mask_out + (size_t)n * Tc : NULL,
                  margin_out ? margin_out + (size_t)n * Tc : NULL, cn,
                  traj ? traj + (size_t)n * Tc * block_m * 2 : NULL);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* One query block of the appendix's sparse-attention variants, all built on plain online softmax
 * (key blocks in ascending order, exact-max update on every block, no seed):
 *   skip     1 = the BLASST test before every block (vanilla BLASST): drop the block iff
 *            m~ - max(m, m~) < ln(lambda) for all rows
 *   rowskip  Blasst_Rowskip: in a block that is kept, a row that fails the same test contributes
 *            nothing (zero mass) and its state does not move
 *   lazy_tau >= 0: Blasst_FA4's rescale-skip rule: a row adopts the new max only when it exceeds
 *            the old one by more than lazy_tau * ln 2; otherwise it keeps the old max (scale factor 1)
 * Shares only score(), the row accessors and the block geometry with one_block.
 * counters: [0] blocks visited, [1] row-max executions, [2] blocks whose rescale chain ran (rowskip:
 * rows suppressed instead, a skipped block counting all its rows), [3] blocks skipped.            */
static void one_block_variant(const prob_t *p, int skip, double ln_lambda, int rowskip, double lazy_tau,
                              int b, int h, int i, double *O, double *LSE, uint8_t *mask_row,
                              double *margin_row, int64_t *counters) {
    const int N = p->N, d = p->d, Br = p->block_m, Bc = p->block_n;
    const int Tc = ceil_div(N, Bc);
    const int r0 = i * Br, nr = imin(Br, N - r0);
    int a_lo, a_hi, j_hi;
    geometry(N, Br, Bc, p->causal, i, &a_lo, &a_hi, &j_hi);
    double *m = (double *)malloc((size_t)Br * sizeof(double));
    double *l = (double *)calloc((size_t)Br, sizeof(double));
    double *acc = (double *)calloc((size_t)Br * d, sizeof(double));
    double *S = (double *)malloc((size_t)Br * Bc * sizeof(double));
    double *mt = (double *)malloc((size_t)Br * sizeof(double));
    int *live = (int *)malloc((size_t)Br * sizeof(int)); /* row takes part in this block */
    for (int rr = 0; rr < Br; ++rr) m[rr] = -INFINITY;
    if (mask_row) for (int j = 0; j < Tc; ++j) mask_row[j] = 2;
    if (margin_row) for (int j = 0; j < Tc; ++j) margin_row[j] = NAN;

    for (int j = 0; j <= j_hi; ++j) {
        const int c0 = j * Bc, nc = imin(Bc, N - c0);
        for (int rr = 0; rr < nr; ++rr) {
            double x = -INFINITY;
            for (int cc = 0; cc < nc; ++cc) {
                const int r = r0 + rr, c = c0 + cc;
                const double sc = (p->causal && c > r) ? -INFINITY : score(p, b, h, r, c);
                S[rr * Bc + cc] = sc;
                x = fmax(x, sc);
            }
            mt[rr] = x;
            live[rr] = 1;
        }
        counters[0] += 1;
        counters[1] += 1;
        if (skip) {
            double worst = -INFINITY;
            for (int rr = 0; rr < nr; ++rr) {
                const double diff = (mt[rr] == -INFINITY) ? -INFINITY : mt[rr] - fmax(m[rr], mt[rr]);
                if (rowskip && diff < ln_lambda) live[rr] = 0;
                worst = fmax(worst, diff);
            }
            if (margin_row) margin_row[j] = worst - ln_lambda;
            if (worst < ln_lambda) {
                if (mask_row) mask_row[j] = 1;
                counters[3] += 1;
                if (rowskip) counters[2] += nr;
                continue;
            }
            if (rowskip)
                for (int rr = 0; rr < nr; ++rr) counters[2] += live[rr] ? 0 : 1;
        }
        if (mask_row) mask_row[j] = 0;
        int rescaled = 0;
        for (int rr = 0; rr < nr; ++rr) {
            if (!live[rr]) continue;
            double m_new = fmax(m[rr], mt[rr]);
            if (lazy_tau >= 0.0 && m[rr] != -INFINITY && m_new - m[rr] <= lazy_tau * 0.69314718055994530942)
                m_new = m[rr]; /* the max grew too little to be worth a rescale */
            if (m_new != m[rr]) rescaled = 1;
            const double alpha = (m_new == -INFINITY) ? 1.0 : exp(m[rr] - m_new);
            double *orow = acc + (size_t)rr * d;
            for (int t = 0; t < d; ++t) orow[t] *= alpha;
            l[rr] *= alpha;
            double rowsum = 0.0;
            for (int cc = 0; cc < nc; ++cc) {
                const double sc = S[rr * Bc + cc];
                const double pt = (sc == -INFINITY) ? 0.0 : exp(sc - m_new);
                rowsum += pt;
                const float *v = v_row(p, b, h, c0 + cc);
                for (int t = 0; t < d; ++t) orow[t] += pt * (double)v[t];
            }
            l[rr] += rowsum; /* (the block's mass first, then onto l: the order of Table 1's rowsum step) */
            m[rr] = m_new;
        }
        if (!rowskip) counters[2] += (lazy_tau >= 0.0) ? rescaled : 1;
    }
    for (int rr = 0; rr < nr; ++rr) {
        for (int t = 0; t < d; ++t) O[(size_t)rr * d + t] = (l[rr] > 0.0) ? acc[(size_t)rr * d + t] / l[rr] : 0.0;
        LSE[rr] = (l[rr] > 0.0) ? m[rr] + log(l[rr]) : -INFINITY;
    }
    free(m); free(l); free(acc); free(S); free(mt); free(live);
}

/* Online softmax with the conditional rescale of the "Blasst_FA4" variant (its second stage
 * alone, no block skipping): ascending order, row max on every block, but a row adopts the
 * new max only when it exceeds the old one by more than tau * ln 2; otherwise the old max is
 * used and the row's scale factor is exactly 1.  The result is the exact attention output for
 * any tau >= 0 (the max cancels in O / l); what changes is how often the rescale runs.
 *   counters [nblk, 4]: tiles visited, rowmax executions, tiles whose rescale chain ran, 0   */
int oracle_fa_lazy(const float *Q, const float *K, const float *V, int B, int Hq, int Hkv, int N,
                   int d, int block_m, int block_n, int causal, double scale, double tau, int nblk,
                   const int *blocks, double *O, double *LSE, int64_t *counters) {
    if (Hq % Hkv != 0 || block_m <= 0 || block_n <= 0 || !(tau >= 0.0)) return -1;
    prob_t p = {Q, K, V, B, Hq, Hkv, N, d, block_m, block_n, causal, scale};
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < nblk; ++n) {
        int64_t *cn = counters + (size_t)n * 4;
        cn[0] = cn[1] = cn[2] = cn[3] = 0;
        one_block_variant(&p, 0, 0.0, 0, tau, blocks[3 * n], blocks[3 * n + 1], blocks[3 * n + 2],
                          O + (size_t)n * block_m * d, LSE + (size_t)n * block_m, NULL, NULL, cn);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Decode step against a key/value cache (Step 1: summaries of a growing cache are extended block
 * by block; the rest is Alg. 1 with a query block of one token per head that sees every key).
 *   q [B,Hq,d]; K, V [B,Hkv,n_cap,d] of which the first n_keys rows are valid
 *   krepr [B,Hkv,ceil(n_keys/block_n),d] or NULL (then m_init = -inf)
 *   O [B,Hq,d], LSE [B,Hq]: the plain definition over keys 0..n_keys-1, two passes
 *   m_init [B,Hq]: max_j scale * q . krepr_j over all blocks of the cache
 *   m_final [B,Hq]: max(m_init, exact max over the keys of the first n_sink blocks and of the
 *     last n_local blocks): the value Alg. 1's max holds once its sink / local blocks are done,
 *     and the one a split of the remaining blocks over several workers can share.
 * Because every later block is accumulated against m_final with no further update, the partial
 * (sum exp(s - m_final) v, sum exp(s - m_final)) of disjoint key ranges ADD: l_parts [B,Hq,n_parts]
 * returns the second of these for n_parts equal ranges of whole blocks so that a test can check
 * that they sum to exp(LSE - m_final).                                                     */
int oracle_decode(const float *q, const float *K, const float *V, int B, int Hq, int Hkv, int n_cap,
                  int n_keys, int d, int block_n, double scale, int n_sink, int n_local,
                  const double *krepr, int n_parts, double *O, double *LSE, double *m_init,
                  double *m_final, double *l_parts) {
    if (Hq % Hkv != 0 || n_keys < 1 || n_keys > n_cap || block_n <= 0 || n_parts < 1) return -1;
    const int g = Hq / Hkv, Tc = ceil_div(n_keys, block_n);
    const int per = ceil_div(Tc, n_parts);
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * Hq; ++bh) {
        const int b = bh / Hq, h = bh % Hq, hkv = h / g;
        const float *qr = q + (size_t)bh * d;
        const float *Kh = K + ((size_t)b * Hkv + hkv) * n_cap * d;
        const float *Vh = V + ((size_t)b * Hkv + hkv) * n_cap * d;
        double *s = (double *)malloc((size_t)n_keys * sizeof(double));
        double mx = -INFINITY, sum = 0.0;
        for (int c = 0; c < n_keys; ++c) {
            double a = 0.0;
            for (int t = 0; t < d; ++t) a += (double)qr[t] * (double)Kh[(size_t)c * d + t];
            s[c] = scale * a;
            mx = fmax(mx, s[c]);
        }
        double mi = -INFINITY;
        if (krepr)
            for (int j = 0; j < Tc; ++j) {
                const double *kr = krepr + (((size_t)b * Hkv + hkv) * Tc + j) * d;
                double a = 0.0;
                for (int t = 0; t < d; ++t) a += (double)qr[t] * kr[t];
                mi = fmax(mi, scale * a);
            }
        double mf = mi;
        for (int j = 0; j < Tc; ++j)
            if (j < n_sink || j >= Tc - n_local)
                for (int c = j * block_n; c < imin(n_keys, (j + 1) * block_n); ++c) mf = fmax(mf, s[c]);
        if (l_parts)
            for (int part = 0; part < n_parts; ++part) {
                double lp = 0.0;
                for (int c = part * per * block_n; c < imin(n_keys, (part + 1) * per * block_n); ++c)
                    lp += exp(s[c] - mf);
                l_parts[(size_t)bh * n_parts + part] = lp;
            }
        double *o = O + (size_t)bh * d;
        for (int t = 0; t < d; ++t) o[t] = 0.0;
        for (int c = 0; c < n_keys; ++c) {
            const double pc = exp(s[c] - mx);
            sum += pc;
            for (int t = 0; t < d; ++t) o[t] += pc * (double)Vh[(size_t)c * d + t];
        }
        for (int t = 0; t < d; ++t) o[t] /= sum;
        LSE[bh] = mx + log(sum);
        if (m_init) m_init[bh] = mi;
        if (m_final) m_final[bh] = mf;
        free(s);
    }
    return 0;
}

/* The two remaining skip variants of the appendix, both in ascending order with the exact-max
 * update on every block and no m-init (as vanilla BLASST):
 *   rowskip = 1  Blasst_Rowskip: a tile is skipped only if no row passes the threshold test; in a
 *                kept tile the rows that fail it are suppressed (scores -inf, state untouched).
 *                counters[2] = suppressed rows (the variant's row-wise sparsity numerator)
 *   lazy_tau >= 0  Blasst_FA4: block skip first, then on kept tiles a row keeps its old max while
 *                the new one exceeds it by at most lazy_tau * ln 2.  counters[2] = tiles whose
 *                rescale chain ran
 * counters [nblk, 4] as in oracle_blocks otherwise; mask_out / margin_out as there.            */
int oracle_blasst_variant(const float *Q, const float *K, const float *V, int B, int Hq, int Hkv,
                          int N, int d, int block_m, int block_n, int causal, double scale,
                          double ln_lambda, int rowskip, double lazy_tau, int nblk, const int *blocks,
                          double *O, double *LSE, uint8_t *mask_out, double *margin_out,
                          int64_t *counters) {
    if (Hq % Hkv != 0 || block_m <= 0 || block_n <= 0 || !(ln_lambda < 0.0)) return -1;
    if (rowskip && lazy_tau >= 0.0) return -1;
    prob_t p = {Q, K, V, B, Hq, Hkv, N, d, block_m, block_n, causal, scale};
    const int Tc = ceil_div(N, block_n);
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < nblk; ++n) {
        int64_t *cn = counters + (size_t)n * 4;
        cn[0] = cn[1] = cn[2] = cn[3] = 0;
        one_block_variant(&p, 1, ln_lambda, rowskip, lazy_tau, blocks[3 * n], blocks[3 * n + 1], blocks[3 * n + 2],
                          O + (size_t)n * block_m * d, LSE + (size_t)n * block_m,
                          mask_out ? mask_out + (size_t)n * Tc : NULL,
                          margin_out ? margin_out + (size_t)n * Tc : NULL, cn);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* FP8 (OCP E4M3, finite-only: bias 7, 3 mantissa bits, largest finite 448, no infinities;
 * the published format) for the 8-bit tensor regime of the performance discussion (C8V32).
 * code = round-to-nearest-even of x * inv_scale (the product taken in float32, as the GPU
 * pre-pass takes it), saturated to +-448; NaN -> 0x7F.  Subnormals: multiples of 2^-9.       */
static uint8_t e4m3_encode(float xf) {
    if (xf != xf) return 0x7F;
    uint8_t sign = (xf < 0.0f || (xf == 0.0f && 1.0f / xf < 0.0f)) ? 0x80 : 0x00;
    double a = fabs((double)xf);
    if (a >= 448.0) return sign | 0x7E;                  /* saturate to the largest finite value */
    if (a < 0.015625) {                                  /* below 2^-6: subnormal grid, step 2^-9 */
        double q = a * 512.0;
        double r = nearbyint(q);                         /* default rounding mode: nearest even */
        return sign | (uint8_t)r;                        /* r == 8 is exactly code 0x08 = 2^-6 */
    }
    int e;
    double f = frexp(a, &e);                             /* a = f * 2^e, f in [0.5, 1) */
    double m = f * 2.0;                                  /* [1, 2) */
    int ex = e - 1;
    double r = nearbyint((m - 1.0) * 8.0);               /* 0..8 */
    if (r == 8.0) { r = 0.0; ex += 1; }
    if (ex > 8 || (ex == 8 && r > 6.0)) return sign | 0x7E;
    return sign | (uint8_t)(((ex + 7) << 3) | (int)r);
}

static double e4m3_decode(uint8_t c) {
    const int s = c >> 7, e = (c >> 3) & 15, m = c & 7;
    if (e == 15 && m == 7) return NAN;
    const double v = (e == 0) ? ldexp((double)m, -9) : ldexp(1.0 + m / 8.0, e - 7);
    return s ? -v : v;
}

int oracle_e4m3_quantize(const float *x, long long n, float inv_scale, uint8_t *codes) {
    for (long long i = 0; i < n; ++i) codes[i] = e4m3_encode(x[i] * inv_scale);
    return 0;
}

int oracle_e4m3_dequantize(const uint8_t *codes, long long n, double scale, double *out) {
    for (long long i = 0; i < n; ++i) out[i] = e4m3_decode(codes[i]) * scale;
    return 0;
}

/* ------------------------------------------------------------------ */
/* Microscaling (MX) block formats for the 4-bit tensor regime of the performance discussion (the
 * "C4" configurations): the published OCP MX layout, 32 consecutive elements along the feature
 * axis share one E8M0 scale 2^(byte - 127); the elements are
 *   fmt 0  E2M1 (bias 1, one mantissa bit: 0, 0.5, 1, 1.5, 2, 3, 4, 6 and their negatives), two
 *          to a byte, element 2i in the low nibble of byte i;
 *   fmt 1  E5M2 (bias 15, two mantissa bits, largest finite 57344), one to a byte; used for the
 *          key-block summaries of E2M1 keys, whose entries carry different scales.
 * Shared scale (the MX rule): byte = floor(log2(max|x|)) - emax + 127 with emax = 2 (E2M1) or 15
 * (E5M2), clamped to [0, 254]; a block of zeros gets byte 0.  Elements: x / 2^(byte - 127) rounded
 * to the nearest representable value, ties to the even mantissa, saturated at the largest finite
 * value (the formats' infinities and NaNs are never produced).                                  */
static unsigned minifloat_encode(double a, int mb, int bias, double maxv, unsigned maxcode) {
    if (a >= maxv) return maxcode;
    if (a < ldexp(1.0, 1 - bias))                          /* subnormal grid, step 2^(1 - bias - mb) */
        return (unsigned)nearbyint(ldexp(a, mb - 1 + bias)); /* reaching 2^mb is the first normal code */
    int e;
    double f = frexp(a, &e);                               /* a = (2 f) 2^(e - 1), 2 f in [1, 2) */
    int ex = e - 1;
    double r = nearbyint((2.0 * f - 1.0) * (double)(1 << mb));
    if (r == (double)(1 << mb)) { r = 0.0; ex += 1; }
    unsigned code = ((unsigned)(ex + bias) << mb) | (unsigned)r;
    return code > maxcode ? maxcode : code;
}

static double minifloat_decode(unsigned mag, int mb, int bias) {
    const unsigned e = mag >> mb, m = mag & ((1u << mb) - 1u);
    return e == 0 ? ldexp((double)m, 1 - bias - mb) : ldexp(1.0 + (double)m / (double)(1 << mb), (int)e - bias);
}

/* x [rows, d] float32, d a multiple of 32; y = x * pre_scale is taken in float32 (as the GPU
 * pre-pass takes it).  codes: fmt 0 [rows, d/2], fmt 1 [rows, d]; scales [rows, d/32].       */
int oracle_mx_quantize(const float *x, long long rows, int d, float pre_scale, int fmt,
                       uint8_t *codes, uint8_t *scales) {
    if (d <= 0 || d % 32 != 0 || (fmt != 0 && fmt != 1)) return -1;
    const int mb = fmt ? 2 : 1, bias = fmt ? 15 : 1, emax = fmt ? 15 : 2, sbit = fmt ? 0x80 : 0x8;
    const double maxv = fmt ? 57344.0 : 6.0;
    const unsigned maxcode = fmt ? 0x7B : 0x7;
    for (long long r = 0; r < rows; ++r)
        for (int g = 0; g < d / 32; ++g) {
            float y[32];
            double amax = 0.0;
            for (int t = 0; t < 32; ++t) {
                y[t] = x[r * d + 32 * g + t] * pre_scale;
                amax = fmax(amax, fabs((double)y[t]));
            }
            int byte = 0;
            if (amax > 0.0) {
                int e;
                (void)frexp(amax, &e);                     /* floor(log2(amax)) = e - 1 */
                byte = (e - 1) - emax + 127;
                if (byte < 0) byte = 0;
                if (byte > 254) byte = 254;
            }
            scales[r * (d / 32) + g] = (uint8_t)byte;
            for (int t = 0; t < 32; ++t) {
                const double v = ldexp((double)y[t], 127 - byte);
                unsigned c = minifloat_encode(fabs(v), mb, bias, maxv, maxcode);
                if (v < 0.0 || (v == 0.0 && signbit(v))) c |= (unsigned)sbit;
                const long long idx = r * d + 32 * g + t;
                if (fmt) codes[idx] = (uint8_t)c;
                else if (idx & 1) codes[idx >> 1] |= (uint8_t)(c << 4);
                else codes[idx >> 1] = (uint8_t)c;
            }
        }
    return 0;
}

int oracle_mx_dequantize(const uint8_t *codes, const uint8_t *scales, long long rows, int d, int fmt,
                         double *out) {
    if (d <= 0 || d % 32 != 0 || (fmt != 0 && fmt != 1)) return -1;
    for (long long r = 0; r < rows; ++r)
        for (int t = 0; t < d; ++t) {
            const long long idx = r * d + t;
            const unsigned c = fmt ? codes[idx] : ((codes[idx >> 1] >> (4 * (idx & 1))) & 0xF);
            const unsigned sbit = fmt ? 0x80 : 0x8;
            const double v = minifloat_decode(c & (sbit - 1), fmt ? 2 : 1, fmt ? 15 : 1);
            out[idx] = ldexp((c & sbit) ? -v : v, (int)scales[r * (d / 32) + t / 32] - 127);
        }
    return 0;
}
