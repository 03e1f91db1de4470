/*
 * sta_oracle.c -- plain, slow, fp64 CPU oracle for Sliding Tile Attention (STA).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the independent checker for the HIP
 * path: it shares no code, header, table or helper with the GPU library and
 * must only be used from the tests, the smoke check and the benchmark's
 * cpu_baseline leg.  It is written for clarity, not speed, and is never tuned.
 *
 * What it computes, all in raster token order (no tiling anywhere in the
 * attention itself, so a permutation mistake on the GPU side cannot cancel):
 *
 *   - sta_oracle_keep:      the STA mask predicate of one (query token, key
 *                           token) pair -- appendix algorithm "Mask Definition
 *                           of 3D STA".
 *   - sta_oracle_attention: masked softmax attention, Eq. 1 of the paper
 *                           (S = QK^T/sqrt(d_k), A = softmax(S+M), O = AV) with
 *                           M_ij = 0 where the predicate holds and -inf
 *                           elsewhere, evaluated token by token over ALL N
 *                           keys (brute force), fp64 arithmetic.
 *   - sta_oracle_attention_lse: the same plus log(sum_j exp(S_ij + M_ij)) per row.
 *   - sta_oracle_probs:     one row of A (for the "rows sum to 1" invariant).
 *   - sta_oracle_attention_backward: gradients of Eq. 1 with the same mask
 *                           with respect to Q, K and V for a given upstream
 *                           gradient of O (what finetuning through STA,
 *                           Sec. 3.2, differentiates).  The paper prints no
 *                           backward formula; this is the chain rule applied
 *                           to Eq. 1, step by step, in fp64.
 *   - sta_oracle_tile_order / _tile_permute / _untile:
 *                           the tile-contiguous token order of Sec. 3.1 (the
 *                           tokens of a tile occupy one run of the sequence)
 *                           and appendix "Tiling in STA".
 *   - sta_oracle_key_tiles: key-tile list of every query tile, obtained by
 *                           collapsing the token predicate (first token of
 *                           each tile).
 *   - sta_oracle_block_census: dense / mixed / empty classification of every
 *                           (query tile, key tile) block by brute force over
 *                           all its token pairs (Sec. 2.2 taxonomy, Theorem 2).
 *   - sta_oracle_natten_keep: the sliding-window predicate the paper compares
 *                           against -- appendix algorithm "Mask Definition of
 *                           3D NATTEN" (window centre shifted inward at the
 *                           borders, token granularity).
 *   - sta_oracle_block_census_per_query: the same classification for either
 *                           predicate and for either token order (tile-
 *                           contiguous blocks = "tiled", or blocks of
 *                           consecutive raster tokens), one count pair per
 *                           query block (Sec. 2.2; Theorems 1 and 2; Table 1).
 *
 * Readings of the paper taken here (each also listed in the design notes):
 *   - "W_tile / 2" in the mask algorithm is integer floor division.
 *   - Tile ids run row-major over (tile_t, tile_h, tile_w); tokens inside a
 *     tile run row-major over (i_t, i_h, i_w); slot = tile_id * P + intra_id.
 *   - The window is given in tokens (the algorithm's "kernel size"), and is
 *     converted to tiles by floor division as the algorithm states.
 *
 * Inputs are float32 arrays holding the user's exact values (bf16 and fp32
 * are both exactly representable); every arithmetic step widens to double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------------- */
/* Mask predicate: appendix algorithm "Mask Definition of 3D STA".          */
/* q, k: token coordinates (t, h, w); L: video size; W: window ("kernel")   */
/* size in tokens; T: tile size.  Returns 1 if the key is kept.             */
/* ---------------------------------------------------------------------- */
static int imin(int a, int b) { return a < b ? a : b; }
static int imax(int a, int b) { return a > b ? a : b; }

int sta_oracle_keep(const int q[3], const int k[3], const int L[3],
                    const int W[3], const int T[3])
{
    int keep = 1;
    for (int a = 0; a < 3; ++a) {
        /* QK coordinates in tiles */
        int q_tile = q[a] / T[a];
        int k_tile = k[a] / T[a];
        /* window size in tiles */
        int W_tile = W[a] / T[a];
        /* half window, integer floor (reading: the printed fraction is //) */
        int half = W_tile / 2;
        /* window centre: min first, max applied last */
        int q_c = imax(imin(q_tile, (L[a] / T[a] - 1) - half), half);
        /* per-axis constraint */
        int constraint = abs(q_c - k_tile) <= half;
        keep = keep && constraint;
    }
    return keep;
}

static void unravel(long i, const int L[3], int c[3])
{
    c[2] = (int)(i % L[2]);
    c[1] = (int)((i / L[2]) % L[1]);
    c[0] = (int)(i / ((long)L[2] * L[1]));
}

/* ---------------------------------------------------------------------- */
/* Masked attention, Eq. 1, for ONE head.                                   */
/* q, k, v: [N, d] float32, raster order, N = L[0]*L[1]*L[2].               */
/* query_idx[nq]: raster indices of the query tokens to evaluate.           */
/* out: [nq, d] double.  scale multiplies QK^T (Eq. 1: 1/sqrt(d_k)).        */
/* srow: caller-provided scratch of N doubles.                              */
/* ---------------------------------------------------------------------- */
static void attention_one_query(const float *q, const float *k, const float *v,
                                long N, int d, const int L[3], const int W[3],
                                const int T[3], double scale, long i,
                                double *srow, double *out_row, double *row_sum,
                                double *lse)
{
    int qc[3], kc[3];
    unravel(i, L, qc);
    /* S + M : one full row over every key token */
    double m = -INFINITY;
    for (long j = 0; j < N; ++j) {
        unravel(j, L, kc);
        if (sta_oracle_keep(qc, kc, L, W, T)) {
            double dot = 0.0;
            for (int c = 0; c < d; ++c)
                dot += (double)q[i * d + c] * (double)k[j * d + c];
            srow[j] = dot * scale;           /* M_ij = 0 */
        } else {
            srow[j] = -INFINITY;             /* M_ij = -inf */
        }
        if (srow[j] > m) m = srow[j];
    }
    /* A = softmax(S + M) */
    double denom = 0.0;
    for (long j = 0; j < N; ++j) {
        srow[j] = exp(srow[j] - m);          /* exp(-inf) = 0 */
        denom += srow[j];
    }
    /* log of the softmax denominator, log(sum_j exp(S_ij + M_ij)) */
    if (lse) *lse = m + log(denom);
    for (long j = 0; j < N; ++j) srow[j] /= denom;
    /* O = A V */
    if (out_row) {
        for (int c = 0; c < d; ++c) out_row[c] = 0.0;
        for (long j = 0; j < N; ++j) {
            if (srow[j] == 0.0) continue;
            for (int c = 0; c < d; ++c)
                out_row[c] += srow[j] * (double)v[j * d + c];
        }
    }
    if (row_sum) {
        double s = 0.0;
        for (long j = 0; j < N; ++j) s += srow[j];
        *row_sum = s;
    }
}

/* lse (optional, [nq]): natural log of the softmax denominator of each query row. */
int sta_oracle_attention_lse(const float *q, const float *k, const float *v,
                             int d, const int L[3], const int T[3], const int W[3],
                             double scale, const int64_t *query_idx, long nq,
                             double *out, double *lse)
{
    long N = (long)L[0] * L[1] * L[2];
    int failed = 0;
#pragma omp parallel
    {
        double *srow = (double *)malloc(sizeof(double) * (size_t)N);
        if (!srow) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 4)
            for (long n = 0; n < nq; ++n)
                attention_one_query(q, k, v, N, d, L, W, T, scale,
                                    (long)query_idx[n], srow, out + n * d, NULL,
                                    lse ? lse + n : NULL);
        }
        free(srow);
    }
    return failed ? -1 : 0;
}

int sta_oracle_attention(const float *q, const float *k, const float *v,
                         int d, const int L[3], const int T[3], const int W[3],
                         double scale, const int64_t *query_idx, long nq,
                         double *out)
{
    return sta_oracle_attention_lse(q, k, v, d, L, T, W, scale, query_idx, nq, out, NULL);
}

/* ---------------------------------------------------------------------- */
/* Gradients of Eq. 1 (same mask) for ONE head, raster order.               */
/* Forward:  S = Q K^T * scale,  A = softmax(S + M) row-wise,  O = A V.      */
/* Given G = dLoss/dO, the chain rule gives, for kept pairs (i, j):         */
/*   dV_j  = sum_i A_ij G_i                       (O is linear in V)        */
/*   dA_ij = G_i . V_j                                                      */
/*   dS_ij = A_ij (dA_ij - sum_l A_il dA_il)      (softmax Jacobian)        */
/*         = A_ij (dA_ij - G_i . O_i)                                       */
/*   dQ_i  = scale * sum_j dS_ij K_j,   dK_j = scale * sum_i dS_ij Q_i.     */
/* Masked pairs have A_ij = 0 and contribute nothing.                       */
/* dq is returned for the rows in query_idx, dk and dv for the rows in      */
/* key_idx (each still summed over ALL partners by brute force).            */
/* ---------------------------------------------------------------------- */
int sta_oracle_attention_backward(const float *q, const float *k, const float *v,
                                  const float *g, int d, const int L[3],
                                  const int T[3], const int W[3], double scale,
                                  const int64_t *query_idx, long nq,
                                  const int64_t *key_idx, long nk,
                                  double *dq, double *dk, double *dv)
{
    long N = (long)L[0] * L[1] * L[2];
    /* Row statistics are needed for the queries asked for and for every query
     * that keeps one of the keys asked for. */
    unsigned char *need = (unsigned char *)calloc((size_t)N, 1);
    double *row_max = (double *)malloc(sizeof(double) * (size_t)N);
    double *row_den = (double *)malloc(sizeof(double) * (size_t)N);
    double *row_go = (double *)malloc(sizeof(double) * (size_t)N);   /* G_i . O_i */
    if (!need || !row_max || !row_den || !row_go) {
        free(need); free(row_max); free(row_den); free(row_go);
        return -1;
    }
    for (long n = 0; n < nq; ++n) need[query_idx[n]] = 1;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < N; ++i) {
        int qc[3], kc[3];
        unravel(i, L, qc);
        for (long n = 0; n < nk && !need[i]; ++n) {
            unravel((long)key_idx[n], L, kc);
            if (sta_oracle_keep(qc, kc, L, W, T)) need[i] = 1;
        }
    }
    int failed = 0;
#pragma omp parallel
    {
        double *srow = (double *)malloc(sizeof(double) * (size_t)N);
        double *orow = (double *)malloc(sizeof(double) * (size_t)d);
        if (!srow || !orow) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
            /* forward rows: max, denominator, G_i . O_i */
#pragma omp for schedule(dynamic, 4)
            for (long i = 0; i < N; ++i) {
                if (!need[i]) continue;
                int qc[3], kc[3];
                unravel(i, L, qc);
                double m = -INFINITY;
                for (long j = 0; j < N; ++j) {
                    unravel(j, L, kc);
                    if (sta_oracle_keep(qc, kc, L, W, T)) {
                        double dot = 0.0;
                        for (int c = 0; c < d; ++c) dot += (double)q[i * d + c] * (double)k[j * d + c];
                        srow[j] = dot * scale;
                        if (srow[j] > m) m = srow[j];
                    } else {
                        srow[j] = -INFINITY;
                    }
                }
                double den = 0.0;
                for (long j = 0; j < N; ++j) den += exp(srow[j] - m);
                for (int c = 0; c < d; ++c) orow[c] = 0.0;
                for (long j = 0; j < N; ++j) {
                    if (srow[j] == -INFINITY) continue;
                    double a = exp(srow[j] - m) / den;
                    for (int c = 0; c < d; ++c) orow[c] += a * (double)v[j * d + c];
                }
                double go = 0.0;
                for (int c = 0; c < d; ++c) go += (double)g[i * d + c] * orow[c];
                row_max[i] = m; row_den[i] = den; row_go[i] = go;
            }
            /* dQ rows */
#pragma omp for schedule(dynamic, 4)
            for (long n = 0; n < nq; ++n) {
                long i = (long)query_idx[n];
                int qc[3], kc[3];
                unravel(i, L, qc);
                for (int c = 0; c < d; ++c) dq[n * d + c] = 0.0;
                for (long j = 0; j < N; ++j) {
                    unravel(j, L, kc);
                    if (!sta_oracle_keep(qc, kc, L, W, T)) continue;
                    double dot = 0.0, da = 0.0;
                    for (int c = 0; c < d; ++c) {
                        dot += (double)q[i * d + c] * (double)k[j * d + c];
                        da += (double)g[i * d + c] * (double)v[j * d + c];
                    }
                    double a = exp(dot * scale - row_max[i]) / row_den[i];
                    double ds = a * (da - row_go[i]);
                    for (int c = 0; c < d; ++c) dq[n * d + c] += scale * ds * (double)k[j * d + c];
                }
            }
            /* dK and dV rows */
#pragma omp for schedule(dynamic, 1)
            for (long n = 0; n < nk; ++n) {
                long j = (long)key_idx[n];
                int qc[3], kc[3];
                unravel(j, L, kc);
                for (int c = 0; c < d; ++c) { dk[n * d + c] = 0.0; dv[n * d + c] = 0.0; }
                for (long i = 0; i < N; ++i) {
                    unravel(i, L, qc);
                    if (!sta_oracle_keep(qc, kc, L, W, T)) continue;
                    double dot = 0.0, da = 0.0;
                    for (int c = 0; c < d; ++c) {
                        dot += (double)q[i * d + c] * (double)k[j * d + c];
                        da += (double)g[i * d + c] * (double)v[j * d + c];
                    }
                    double a = exp(dot * scale - row_max[i]) / row_den[i];
                    double ds = a * (da - row_go[i]);
                    for (int c = 0; c < d; ++c) {
                        dv[n * d + c] += a * (double)g[i * d + c];
                        dk[n * d + c] += scale * ds * (double)q[i * d + c];
                    }
                }
            }
        }
        free(srow); free(orow);
    }
    free(need); free(row_max); free(row_den); free(row_go);
    return failed ? -1 : 0;
}

/* One row of A (probabilities over all N keys) and its sum. */
int sta_oracle_probs(const float *q, const float *k, int d, const int L[3],
                     const int T[3], const int W[3], double scale, long i,
                     double *probs /* [N] */, double *row_sum)
{
    long N = (long)L[0] * L[1] * L[2];
    attention_one_query(q, k, NULL, N, d, L, W, T, scale, i, probs, NULL,
                        row_sum, NULL);
    return 0;
}

/* ---------------------------------------------------------------------- */
/* Tile-contiguous token order.                                             */
/* order[slot] = raster index of the token stored at tiled slot `slot`.     */
/* Written as the nested coordinate loops themselves.                       */
/* ---------------------------------------------------------------------- */
int sta_oracle_tile_order(const int L[3], const int T[3], int64_t *order)
{
    if (L[0] % T[0] || L[1] % T[1] || L[2] % T[2]) return -1;
    long slot = 0;
    for (int tt = 0; tt < L[0] / T[0]; ++tt)
     for (int th = 0; th < L[1] / T[1]; ++th)
      for (int tw = 0; tw < L[2] / T[2]; ++tw)
       for (int it = 0; it < T[0]; ++it)
        for (int ih = 0; ih < T[1]; ++ih)
         for (int iw = 0; iw < T[2]; ++iw) {
             long t = (long)tt * T[0] + it;
             long h = (long)th * T[1] + ih;
             long w = (long)tw * T[2] + iw;
             order[slot++] = (t * L[1] + h) * L[2] + w;
         }
    return 0;
}

/* src, dst: [outer, N, row_bytes] byte arrays; moves whole token rows. */
int sta_oracle_tile_permute(const unsigned char *src, unsigned char *dst,
                            long outer, long row_bytes, const int L[3],
                            const int T[3])
{
    long N = (long)L[0] * L[1] * L[2];
    int64_t *order = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
    if (!order) return -1;
    if (sta_oracle_tile_order(L, T, order)) { free(order); return -1; }
    for (long o = 0; o < outer; ++o)
        for (long slot = 0; slot < N; ++slot)
            memcpy(dst + (o * N + slot) * row_bytes,
                   src + (o * N + order[slot]) * row_bytes, (size_t)row_bytes);
    free(order);
    return 0;
}

int sta_oracle_untile(const unsigned char *src, unsigned char *dst, long outer,
                      long row_bytes, const int L[3], const int T[3])
{
    long N = (long)L[0] * L[1] * L[2];
    int64_t *order = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
    if (!order) return -1;
    if (sta_oracle_tile_order(L, T, order)) { free(order); return -1; }
    for (long o = 0; o < outer; ++o)
        for (long slot = 0; slot < N; ++slot)
            memcpy(dst + (o * N + order[slot]) * row_bytes,
                   src + (o * N + slot) * row_bytes, (size_t)row_bytes);
    free(order);
    return 0;
}

/* ---------------------------------------------------------------------- */
/* Key-tile lists by collapsing the token predicate: query tile qt keeps    */
/* key tile kt iff the predicate holds for their first tokens.              */
/* counts: [n]; lists: [n][n], ascending row-major tile ids, -1 padded.     */
/* ---------------------------------------------------------------------- */
static void tile_first_token(long tile, const int L[3], const int T[3], int c[3])
{
    int nt[3] = { L[0] / T[0], L[1] / T[1], L[2] / T[2] };
    int tc[3];
    unravel(tile, nt, tc);
    for (int a = 0; a < 3; ++a) c[a] = tc[a] * T[a];
}

int sta_oracle_key_tiles(const int L[3], const int T[3], const int W[3],
                         int32_t *counts, int32_t *lists)
{
    if (L[0] % T[0] || L[1] % T[1] || L[2] % T[2]) return -1;
    long n = (long)(L[0] / T[0]) * (L[1] / T[1]) * (L[2] / T[2]);
    for (long qt = 0; qt < n; ++qt) {
        int qc[3], kc[3];
        tile_first_token(qt, L, T, qc);
        int32_t cnt = 0;
        for (long kt = 0; kt < n; ++kt) {
            tile_first_token(kt, L, T, kc);
            if (sta_oracle_keep(qc, kc, L, W, T)) lists[qt * n + cnt++] = (int32_t)kt;
        }
        counts[qt] = cnt;
        for (long r = cnt; r < n; ++r) lists[qt * n + r] = -1;
    }
    return 0;
}

/* ---------------------------------------------------------------------- */
/* Block census: every (query tile, key tile) block is classified by        */
/* evaluating the predicate on ALL its P x P token pairs.                   */
/* ---------------------------------------------------------------------- */
int sta_oracle_block_census(const int L[3], const int T[3], const int W[3],
                            int64_t *n_dense, int64_t *n_mixed, int64_t *n_empty)
{
    if (L[0] % T[0] || L[1] % T[1] || L[2] % T[2]) return -1;
    long n = (long)(L[0] / T[0]) * (L[1] / T[1]) * (L[2] / T[2]);
    long P = (long)T[0] * T[1] * T[2];
    int64_t dense = 0, mixed = 0, empty = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : dense, mixed, empty)
    for (long qt = 0; qt < n; ++qt) {
        int q0[3], k0[3];
        tile_first_token(qt, L, T, q0);
        for (long kt = 0; kt < n; ++kt) {
            tile_first_token(kt, L, T, k0);
            long kept = 0;
            for (long a = 0; a < P; ++a) {
                int qi[3], qc[3];
                unravel(a, T, qi);
                for (int x = 0; x < 3; ++x) qc[x] = q0[x] + qi[x];
                for (long b = 0; b < P; ++b) {
                    int ki[3], kc[3];
                    unravel(b, T, ki);
                    for (int x = 0; x < 3; ++x) kc[x] = k0[x] + ki[x];
                    kept += sta_oracle_keep(qc, kc, L, W, T);
                }
            }
            if (kept == P * P) dense++;
            else if (kept == 0) empty++;
            else mixed++;
        }
    }
    *n_dense = dense; *n_mixed = mixed; *n_empty = empty;
    return 0;
}

/* ---------------------------------------------------------------------- */
/* Sliding-window predicate: appendix algorithm "Mask Definition of 3D     */
/* NATTEN".  Token coordinates throughout; W/2 is integer floor division    */
/* (windows are odd in the paper, e.g. 11: five keys on either side).       */
/* ---------------------------------------------------------------------- */
int sta_oracle_natten_keep(const int q[3], const int k[3], const int L[3],
                           const int W[3])
{
    int keep = 1;
    for (int a = 0; a < 3; ++a) {
        int half = W[a] / 2;
        /* window centre, shifted inward near the borders */
        int q_c = imax(imin(q[a], L[a] - 1 - half), half);
        keep = keep && (abs(q_c - k[a]) <= half);
    }
    return keep;
}

/* ---------------------------------------------------------------------- */
/* Census per query block for either predicate and either token order.      */
/* mask: 0 = STA (needs T), 1 = sliding window (T only shapes the blocks).  */
/* tiled != 0: block b holds the tokens of tile b (tile-contiguous order);  */
/* tiled == 0: block b holds raster tokens [b*P, (b+1)*P), P = T0*T1*T2.    */
/* dense_per_q, mixed_per_q: [number of blocks].                            */
/* ---------------------------------------------------------------------- */
static void block_token(long block, long i, int tiled, const int L[3],
                        const int T[3], int c[3])
{
    if (tiled) {
        int t0[3], ti[3];
        tile_first_token(block, L, T, t0);
        unravel(i, T, ti);
        for (int a = 0; a < 3; ++a) c[a] = t0[a] + ti[a];
    } else {
        long P = (long)T[0] * T[1] * T[2];
        unravel(block * P + i, L, c);
    }
}

int sta_oracle_block_census_per_query(int mask, int tiled, const int L[3],
                                      const int T[3], const int W[3],
                                      int64_t *dense_per_q, int64_t *mixed_per_q)
{
    long N = (long)L[0] * L[1] * L[2];
    long P = (long)T[0] * T[1] * T[2];
    if (tiled && (L[0] % T[0] || L[1] % T[1] || L[2] % T[2])) return -1;
    if (!tiled && N % P) return -1;
    long nb = N / P;
#pragma omp parallel for schedule(dynamic, 1)
    for (long qb = 0; qb < nb; ++qb) {
        int64_t dense = 0, mixed = 0;
        for (long kb = 0; kb < nb; ++kb) {
            long kept = 0;
            for (long a = 0; a < P; ++a) {
                int qc[3], kc[3];
                block_token(qb, a, tiled, L, T, qc);
                for (long b = 0; b < P; ++b) {
                    block_token(kb, b, tiled, L, T, kc);
                    kept += mask == 0 ? sta_oracle_keep(qc, kc, L, W, T)
                                      : sta_oracle_natten_keep(qc, kc, L, W);
                }
            }
            if (kept == P * P) dense++;
            else if (kept != 0) mixed++;
        }
        dense_per_q[qb] = dense;
        mixed_per_q[qb] = mixed;
    }
    return 0;
}

int sta_oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
