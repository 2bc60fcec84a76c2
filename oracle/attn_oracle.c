/*
 * CPU fp64 oracle for scaled-dot-product attention, forward and backward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU
 * kernels are checked against.  It shares no code with the HIP path, and the
 * product library never links, loads or calls it.
 *
 * Everything here is the textbook definition written out with three nested
 * loops per quantity; no tiling, no fusion, no recurrences:
 *
 *   forward  (paper Sec. 2.1, first display):
 *     S = alpha * Q K^T,   P = softmax_rows(S),   O = P V
 *     with the row maximum subtracted before exponentiation, as the same
 *     section states; masked scores (causal, key position > query position)
 *     are excluded from the row altogether.
 *     LSE_i = m_i + ln(sum_j exp(S_ij - m_i)) is the natural-log row
 *     log-sum-exp of the scaled, masked scores (the quantity the forward
 *     pass hands to the backward pass).
 *
 *   backward (paper Sec. 2.1, second display):
 *     dV = P^T dO,  dP = dO V^T,  dS = (diag(p) - p p^T) dp  row by row,
 *     dQ = alpha dS K,  dK = alpha dS^T Q.
 *     The softmax Jacobian is applied literally as dS_ij = P_ij (dP_ij - D_i)
 *     with D_i = sum_j P_ij dP_ij computed from P and dP themselves (NOT from
 *     dO . O), so the oracle does not take the shortcut the GPU path takes.
 *
 *   grouped-query attention (paper Sec. 3.2.3/3.3 mention several query heads
 *     sharing one KV head): query head h reads KV head h / (H / Hkv); dK and
 *     dV of a KV head are the sums over its query heads.
 *
 * Layouts (row-major, contiguous, fp64):
 *   q  [B, Nq, H,   dqk]     k  [B, Nk, Hkv, dqk]    v  [B, Nk, Hkv, dv]
 *   o, d_o [B, Nq, H, dv]    lse [B, H, Nq]
 *   dq like q, dk like k, dv like v.
 *
 * Causal masking: query row i has a position pos_i (q_pos[i] when q_pos is
 * non-NULL, else i); key j is visible iff j <= pos_i.  q_pos lets a test pass
 * a SUBSET of the query rows of a longer sequence (sampled rows of a big
 * problem) without changing any formula.  A row with no visible key is an
 * error (return -2): the method never produces one.
 *
 * Return 0 on success, -1 on bad arguments, -2 on an empty softmax row.
 * Parallelism: OpenMP over (batch, query head, query row) for forward and dQ;
 * over (batch, KV head, key row) for dK/dV.  Each output element is produced
 * by exactly one thread with a fixed summation order, so results do not
 * depend on the thread count.
 *
 * Pins (tests/test_oracle_*.py): identical keys -> mean of V; a dominant logit
 * selects its V row; rows of P sum to 1; q = 0 closed forms; key-shift and
 * permutation invariances; central finite differences of sum(O * dO); a
 * torch-CPU fp64 softmax/autograd cross-check; GQA == MHA with repeated KV.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int bad_args(int B, int H, int Hkv, int Nq, int Nk, int dqk, int dv)
{
    if (B <= 0 || H <= 0 || Hkv <= 0 || Nq <= 0 || Nk <= 0 || dqk <= 0 || dv <= 0) return 1;
    if (H % Hkv != 0) return 1;
    return 0;
}

/* Scaled scores of one query row against keys 0..nvis-1; returns row max. */
static double score_row(const double* qrow, const double* kbase, size_t kstride,
                        int nvis, int dqk, double scale, double* s)
{
    double m = -INFINITY;
    for (int j = 0; j < nvis; ++j) {
        const double* krow = kbase + (size_t)j * kstride;
        double acc = 0.0;
        for (int c = 0; c < dqk; ++c) acc += qrow[c] * krow[c];
        s[j] = scale * acc;
        if (s[j] > m) m = s[j];
    }
    return m;
}

int oracle_attn_fwd(const double* q, const double* k, const double* v,
                    double* o, double* lse,
                    int B, int H, int Hkv, int Nq, int Nk, int dqk, int dv,
                    double scale, int causal, const int* q_pos)
{
    if (!q || !k || !v || !o || !lse || bad_args(B, H, Hkv, Nq, Nk, dqk, dv)) return -1;
    const int G = H / Hkv;
    const size_t kstride = (size_t)Hkv * dqk, vstride = (size_t)Hkv * dv;
    int status = 0;

#pragma omp parallel
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)Nk);
#pragma omp for collapse(3) schedule(dynamic, 8)
        for (int b = 0; b < B; ++b)
            for (int h = 0; h < H; ++h)
                for (int i = 0; i < Nq; ++i) {
                    const int kvh = h / G;
                    const int pos = q_pos ? q_pos[i] : i;
                    int nvis = causal ? pos + 1 : Nk;
                    if (nvis > Nk) nvis = Nk;
                    double* orow = o + (((size_t)b * Nq + i) * H + h) * dv;
                    if (nvis <= 0) {
#pragma omp atomic write
                        status = -2;
                        continue;
                    }
                    const double* qrow = q + (((size_t)b * Nq + i) * H + h) * dqk;
                    const double* kbase = k + ((size_t)b * Nk * Hkv + kvh) * dqk;
                    const double* vbase = v + ((size_t)b * Nk * Hkv + kvh) * dv;
                    const double m = score_row(qrow, kbase, kstride, nvis, dqk, scale, s);
                    double Z = 0.0;
                    for (int j = 0; j < nvis; ++j) {
                        s[j] = exp(s[j] - m);
                        Z += s[j];
                    }
                    for (int c = 0; c < dv; ++c) orow[c] = 0.0;
                    for (int j = 0; j < nvis; ++j) {
                        const double p = s[j] / Z;
                        const double* vrow = vbase + (size_t)j * vstride;
                        for (int c = 0; c < dv; ++c) orow[c] += p * vrow[c];
                    }
                    lse[((size_t)b * H + h) * Nq + i] = m + log(Z);
                }
        free(s);
    }
    return status;
}

int oracle_attn_bwd(const double* q, const double* k, const double* v, const double* d_o,
                    double* dq, double* dk, double* dv_out,
                    int B, int H, int Hkv, int Nq, int Nk, int dqk, int dv,
                    double scale, int causal, const int* q_pos)
{
    if (!q || !k || !v || !d_o || !dq || !dk || !dv_out ||
        bad_args(B, H, Hkv, Nq, Nk, dqk, dv))
        return -1;
    const int G = H / Hkv;
    const size_t kstride = (size_t)Hkv * dqk, vstride = (size_t)Hkv * dv;
    int status = 0;

    /* Row statistics m_i, Z_i and D_i = sum_j P_ij dP_ij, stored so that the
     * dK/dV pass (parallel over key rows) can rebuild P_ij and dS_ij. */
    const size_t nrows = (size_t)B * H * Nq;
    double* rm = (double*)malloc(sizeof(double) * nrows);
    double* rZ = (double*)malloc(sizeof(double) * nrows);
    double* rD = (double*)malloc(sizeof(double) * nrows);
    if (!rm || !rZ || !rD) { free(rm); free(rZ); free(rD); return -1; }

    /* Pass 1: per query row -> P, dP, D, dS, dQ. */
#pragma omp parallel
    {
        double* p = (double*)malloc(sizeof(double) * (size_t)Nk);
        double* dp = (double*)malloc(sizeof(double) * (size_t)Nk);
#pragma omp for collapse(3) schedule(dynamic, 8)
        for (int b = 0; b < B; ++b)
            for (int h = 0; h < H; ++h)
                for (int i = 0; i < Nq; ++i) {
                    const int kvh = h / G;
                    const int pos = q_pos ? q_pos[i] : i;
                    int nvis = causal ? pos + 1 : Nk;
                    if (nvis > Nk) nvis = Nk;
                    const size_t ridx = ((size_t)b * H + h) * Nq + i;
                    double* dqrow = dq + (((size_t)b * Nq + i) * H + h) * dqk;
                    if (nvis <= 0) {
#pragma omp atomic write
                        status = -2;
                        rm[ridx] = 0.0; rZ[ridx] = 1.0; rD[ridx] = 0.0;
                        continue;
                    }
                    const double* qrow = q + (((size_t)b * Nq + i) * H + h) * dqk;
                    const double* dorow = d_o + (((size_t)b * Nq + i) * H + h) * dv;
                    const double* kbase = k + ((size_t)b * Nk * Hkv + kvh) * dqk;
                    const double* vbase = v + ((size_t)b * Nk * Hkv + kvh) * dv;
                    const double m = score_row(qrow, kbase, kstride, nvis, dqk, scale, p);
                    double Z = 0.0;
                    for (int j = 0; j < nvis; ++j) { p[j] = exp(p[j] - m); Z += p[j]; }
                    double D = 0.0;
                    for (int j = 0; j < nvis; ++j) {
                        p[j] /= Z;
                        const double* vrow = vbase + (size_t)j * vstride;
                        double acc = 0.0;
                        for (int c = 0; c < dv; ++c) acc += dorow[c] * vrow[c];
                        dp[j] = acc;
                        D += p[j] * acc;
                    }
                    rm[ridx] = m; rZ[ridx] = Z; rD[ridx] = D;
                    for (int c = 0; c < dqk; ++c) dqrow[c] = 0.0;
                    for (int j = 0; j < nvis; ++j) {
                        const double ds = p[j] * (dp[j] - D);
                        const double* krow = kbase + (size_t)j * kstride;
                        for (int c = 0; c < dqk; ++c) dqrow[c] += ds * krow[c];
                    }
                    for (int c = 0; c < dqk; ++c) dqrow[c] *= scale;
                }
        free(p); free(dp);
    }

    /* Pass 2: per key row -> dK_j = alpha sum_i dS_ij q_i, dV_j = sum_i P_ij dO_i,
     * summed over the query heads of the group in ascending head order. */
#pragma omp parallel for collapse(3) schedule(dynamic, 8)
    for (int b = 0; b < B; ++b)
        for (int kvh = 0; kvh < Hkv; ++kvh)
            for (int j = 0; j < Nk; ++j) {
                double* dkrow = dk + (((size_t)b * Nk + j) * Hkv + kvh) * dqk;
                double* dvrow = dv_out + (((size_t)b * Nk + j) * Hkv + kvh) * dv;
                const double* krow = k + (((size_t)b * Nk + j) * Hkv + kvh) * dqk;
                const double* vrow = v + (((size_t)b * Nk + j) * Hkv + kvh) * dv;
                for (int c = 0; c < dqk; ++c) dkrow[c] = 0.0;
                for (int c = 0; c < dv; ++c) dvrow[c] = 0.0;
                for (int g = 0; g < G; ++g) {
                    const int h = kvh * G + g;
                    for (int i = 0; i < Nq; ++i) {
                        const int pos = q_pos ? q_pos[i] : i;
                        if (causal && j > pos) continue;
                        const size_t ridx = ((size_t)b * H + h) * Nq + i;
                        const double* qrow = q + (((size_t)b * Nq + i) * H + h) * dqk;
                        const double* dorow = d_o + (((size_t)b * Nq + i) * H + h) * dv;
                        double sacc = 0.0, dpacc = 0.0;
                        for (int c = 0; c < dqk; ++c) sacc += qrow[c] * krow[c];
                        for (int c = 0; c < dv; ++c) dpacc += dorow[c] * vrow[c];
                        const double p = exp(scale * sacc - rm[ridx]) / rZ[ridx];
                        const double ds = p * (dpacc - rD[ridx]);
                        for (int c = 0; c < dv; ++c) dvrow[c] += p * dorow[c];
                        for (int c = 0; c < dqk; ++c) dkrow[c] += ds * qrow[c];
                    }
                }
                for (int c = 0; c < dqk; ++c) dkrow[c] *= scale;
            }

    free(rm); free(rZ); free(rD);
    return status;
}

/*
 * Tiled online softmax with thresholded ("conditional") rescaling, in fp64,
 * following the recurrences of paper Sec. 3.1.4: key blocks of `tile` keys
 * are visited in ascending order; a running reference maximum m, a running
 * normaliser l and an un-normalised output accumulator are kept per row; when
 * the block maximum exceeds the reference by more than tau the accumulator
 * and normaliser are multiplied by exp(m_old - m_new) and the reference
 * moves, otherwise the stale reference is kept (second case of the section's
 * case equation).  The final output is accumulator / l and the row
 * log-sum-exp is m_ref + ln(l), both relative to the reference actually used.
 *
 * tau is in natural-log units of the scaled scores (tau = 8 ln 2 corresponds
 * to the section's factor-256 threshold); tau = 0 is the classical online
 * softmax; tau = +inf never rescales after the first block.
 * n_rescale (optional, [B,H,Nq] ints) counts how often each row rescaled
 * after its first block, so tests can see both branches being taken.
 *
 * This function is a second, independent route to the same O and LSE; its
 * agreement with oracle_attn_fwd for every tau is the evidence that the
 * thresholded scheme is exact and that LSE must use the stale reference.
 */
int oracle_attn_fwd_online(const double* q, const double* k, const double* v,
                           double* o, double* lse, int* n_rescale,
                           int B, int H, int Hkv, int Nq, int Nk, int dqk, int dv,
                           double scale, int causal, int tile, double tau)
{
    if (!q || !k || !v || !o || !lse || tile <= 0 || !(tau >= 0.0) ||
        bad_args(B, H, Hkv, Nq, Nk, dqk, dv))
        return -1;
    const int G = H / Hkv;
    const size_t kstride = (size_t)Hkv * dqk, vstride = (size_t)Hkv * dv;

#pragma omp parallel
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)tile);
        double* acc = (double*)malloc(sizeof(double) * (size_t)dv);
#pragma omp for collapse(3) schedule(dynamic, 8)
        for (int b = 0; b < B; ++b)
            for (int h = 0; h < H; ++h)
                for (int i = 0; i < Nq; ++i) {
                    const int kvh = h / G;
                    int nvis = causal ? i + 1 : Nk;
                    if (nvis > Nk) nvis = Nk;
                    const double* qrow = q + (((size_t)b * Nq + i) * H + h) * dqk;
                    const double* kbase = k + ((size_t)b * Nk * Hkv + kvh) * dqk;
                    const double* vbase = v + ((size_t)b * Nk * Hkv + kvh) * dv;
                    double m = -INFINITY, l = 0.0;
                    int nres = 0;
                    for (int c = 0; c < dv; ++c) acc[c] = 0.0;
                    for (int j0 = 0; j0 < nvis; j0 += tile) {
                        const int nb = (nvis - j0 < tile) ? nvis - j0 : tile;
                        const double mb = score_row(qrow, kbase + (size_t)j0 * kstride,
                                                    kstride, nb, dqk, scale, s);
                        if (j0 == 0) {
                            m = mb;                      /* first block fixes the reference */
                        } else if (mb - m > tau) {
                            const double f = exp(m - mb); /* first case: rescale and move */
                            l *= f;
                            for (int c = 0; c < dv; ++c) acc[c] *= f;
                            m = mb;
                            ++nres;
                        }                                /* else: keep the stale reference */
                        for (int j = 0; j < nb; ++j) {
                            const double e = exp(s[j] - m);
                            l += e;
                            const double* vrow = vbase + (size_t)(j0 + j) * vstride;
                            for (int c = 0; c < dv; ++c) acc[c] += e * vrow[c];
                        }
                    }
                    double* orow = o + (((size_t)b * Nq + i) * H + h) * dv;
                    for (int c = 0; c < dv; ++c) orow[c] = acc[c] / l;
                    lse[((size_t)b * H + h) * Nq + i] = m + log(l);
                    if (n_rescale) n_rescale[((size_t)b * H + h) * Nq + i] = nres;
                }
        free(s); free(acc);
    }
    return 0;
}

int oracle_num_threads(void)
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
