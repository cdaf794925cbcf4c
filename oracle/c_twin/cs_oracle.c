/*
 * Plain C twin of the CPU oracle for the calls of one decode step (test infrastructure only).
 *
 * Same definitions as the NumPy oracle beside it, written out as loops in fp64: the measurement
 * operator Phi drawn entry by entry from Philox4x32-10 (Sec. 3, Sec. 8), the sketch y = Phi z, the
 * effective matrix M = Phi Psi with one atom per unit (Sec. 9), block orthogonal matching pursuit
 * over units with a Householder least-squares refit per round (Sec. 8, Sec. 3/7: exactly k units),
 * the block-sparse gated feed-forward layer (Sec. 3, Sec. 7) and head-pruned attention (Sec. 3, Sec. 7).
 * No blocking, no vector intrinsics, no library routine.  Loops over independent tokens / rows carry an
 * OpenMP pragma so that the same code can be timed on one core and on all of them.
 *
 * Pins: tests/test_oracle_c_twin.py checks every function against the NumPy oracle (which carries
 * the pins to the paper and the mathematics) on small and ragged shapes, and the generator against its
 * published known-answer vectors.  Shares nothing with the HIP library; nothing of the product path
 * may call it.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads used by the loops below from now on (n < 1: as many as the runtime offers); returns the count in force. */
int cso_set_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
    else omp_set_num_threads(omp_get_num_procs());
    return n >= 1 ? n : omp_get_num_procs();
#else
    (void)n;
    return 1;
#endif
}

/* ---- Philox4x32-10 (Salmon et al., SC'11): ten rounds, key advanced by two Weyl constants ---- */
void cso_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        if (r > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1; c3 = (uint32_t)p0; c0 = n0; c2 = n2;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Unscaled entry e(row, col) of Phi: ensemble 0 Gaussian (Box-Muller, four normals per call),
 * ensemble 1 Rademacher (128 sign bits per call; bit 0 -> +1, bit 1 -> -1). */
double cso_phi_entry(int ens, uint64_t seed, uint32_t stream, uint32_t row, uint32_t col) {
    const uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
    uint32_t w[4];
    if (ens == 1) {
        const uint32_t ctr[4] = {col / 128u, row, stream, 1u};
        cso_philox4x32_10(ctr, key, w);
        const uint32_t t = col % 128u;
        return ((w[t / 32u] >> (t % 32u)) & 1u) ? -1.0 : 1.0;
    }
    const uint32_t ctr[4] = {col / 4u, row, stream, 0u};
    cso_philox4x32_10(ctr, key, w);
    const uint32_t p = (col % 4u) / 2u;
    const double u1 = ((double)w[2 * p] + 1.0) / 4294967296.0, u2 = ((double)w[2 * p + 1] + 1.0) / 4294967296.0;
    const double rad = sqrt(-2.0 * log(u1)), ang = 2.0 * 3.14159265358979323846 * u2;
    return (col % 2u) ? rad * sin(ang) : rad * cos(ang);
}

/* y[B][m] = Phi z, z[B][n]; columns in ascending order. */
void cso_sketch(int ens, uint64_t seed, uint32_t stream, int m, int n, const double* z, int B, double* y) {
    const double scale = 1.0 / sqrt((double)m);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i) {
        double* acc = (double*)calloc((size_t)B, sizeof(double));
        for (int c = 0; c < n; ++c) {
            const double e = cso_phi_entry(ens, seed, stream, (uint32_t)i, (uint32_t)c);
            for (int t = 0; t < B; ++t) acc[t] += e * z[(size_t)t * n + c];
        }
        for (int t = 0; t < B; ++t) y[(size_t)t * m + i] = acc[t] * scale;
        free(acc);
    }
}

/* M[m][G] = Phi Psi, one atom per unit: psi[G][b] (unit g spreads its coefficient over its b channels),
 * or psi == NULL with b == 1 for the identity dictionary. */
void cso_effective_matrix(int ens, uint64_t seed, uint32_t stream, int m, int G, int b, const double* psi, double* M) {
    const double scale = 1.0 / sqrt((double)m);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i)
        for (int g = 0; g < G; ++g) {
            double s = 0.0;
            for (int c = 0; c < b; ++c)
                s += cso_phi_entry(ens, seed, stream, (uint32_t)i, (uint32_t)(g * b + c)) * (psi ? psi[(size_t)g * b + c] : 1.0);
            M[(size_t)i * G + g] = s * scale;
        }
}

/* Least squares min ||A x - y|| for A [m][K] (row-major, K < m) by Householder QR; A and y are destroyed. */
static void least_squares(double* A, int m, int K, double* y, double* x) {
    for (int j = 0; j < K; ++j) {
        double nrm = 0.0;
        for (int i = j; i < m; ++i) nrm += A[(size_t)i * K + j] * A[(size_t)i * K + j];
        nrm = sqrt(nrm);
        if (nrm == 0.0) continue;
        const double alpha = A[(size_t)j * K + j] > 0.0 ? -nrm : nrm;
        /* v = column j below the diagonal with v_j = a_jj - alpha; H = I - 2 v v^T / (v^T v) */
        A[(size_t)j * K + j] -= alpha;
        double vtv = 0.0;
        for (int i = j; i < m; ++i) vtv += A[(size_t)i * K + j] * A[(size_t)i * K + j];
        if (vtv > 0.0) {
            for (int c = j + 1; c < K; ++c) {
                double dot = 0.0;
                for (int i = j; i < m; ++i) dot += A[(size_t)i * K + j] * A[(size_t)i * K + c];
                const double f = 2.0 * dot / vtv;
                for (int i = j; i < m; ++i) A[(size_t)i * K + c] -= f * A[(size_t)i * K + j];
            }
            double dot = 0.0;
            for (int i = j; i < m; ++i) dot += A[(size_t)i * K + j] * y[i];
            const double f = 2.0 * dot / vtv;
            for (int i = j; i < m; ++i) y[i] -= f * A[(size_t)i * K + j];
        }
        A[(size_t)j * K + j] = alpha;                /* R's diagonal entry; the reflector below it is no longer needed */
    }
    for (int i = K - 1; i >= 0; --i) {
        double s = y[i];
        for (int c = i + 1; c < K; ++c) s -= A[(size_t)i * K + c] * x[c];
        x[i] = s / A[(size_t)i * K + i];
    }
}

/* Block-OMP with one atom per unit on one sketch.  M [m][G], y [m].  normalised: score (m_g^T r)^2 / ||m_g||^2,
 * else (m_g^T r)^2.  Outputs: support[k] ascending, coef[k] in that order (plain refit), ||r||, margin =
 * min over rounds of (best - runner_up) / best.  Returns 0, or -1 for k out of range / k >= m. */
static int block_omp_one(const double* M, int m, int G, const double* y, int k, int normalised,
                         int32_t* support, double* coef, double* resid_norm, double* margin_out) {
    if (k < 1 || k > G || k >= m) return -1;
    double* r = (double*)malloc((size_t)m * sizeof(double));
    double* A = (double*)malloc((size_t)m * k * sizeof(double));
    double* yy = (double*)malloc((size_t)m * sizeof(double));
    double* x = (double*)malloc((size_t)k * sizeof(double));
    double* nrm2 = (double*)malloc((size_t)G * sizeof(double));
    char* taken = (char*)calloc((size_t)G, 1);
    int* chosen = (int*)malloc((size_t)k * sizeof(int));
    for (int g = 0; g < G; ++g) {
        double s = 0.0;
        for (int i = 0; i < m; ++i) s += M[(size_t)i * G + g] * M[(size_t)i * G + g];
        nrm2[g] = s;
    }
    memcpy(r, y, (size_t)m * sizeof(double));
    double margin = 1.0;
    for (int round = 0; round < k; ++round) {
        int best = -1;
        double s1 = -INFINITY, s2 = -INFINITY;
        for (int g = 0; g < G; ++g) {
            if (taken[g]) continue;
            double c = 0.0;
            for (int i = 0; i < m; ++i) c += M[(size_t)i * G + g] * r[i];
            double sc = c * c;
            if (normalised) sc = nrm2[g] > 0.0 ? sc / nrm2[g] : 0.0;
            if (sc > s1) { s2 = s1; s1 = sc; best = g; }          /* first maximum = smallest index */
            else if (sc > s2) s2 = sc;
        }
        if (!(s2 > -INFINITY)) s2 = 0.0;
        if (s1 > 0.0) { const double mg = (s1 - s2) / s1; if (mg < margin) margin = mg; } else margin = 0.0;
        taken[best] = 1;
        chosen[round] = best;
        const int K = round + 1;
        for (int i = 0; i < m; ++i) {
            for (int j = 0; j < K; ++j) A[(size_t)i * K + j] = M[(size_t)i * G + chosen[j]];
            yy[i] = y[i];
        }
        least_squares(A, m, K, yy, x);
        for (int i = 0; i < m; ++i) {
            double s = y[i];
            for (int j = 0; j < K; ++j) s -= M[(size_t)i * G + chosen[j]] * x[j];
            r[i] = s;
        }
    }
    /* ascending support, plain refit in that order */
    int j = 0;
    for (int g = 0; g < G; ++g) if (taken[g]) support[j++] = g;
    for (int i = 0; i < m; ++i) {
        for (int c = 0; c < k; ++c) A[(size_t)i * k + c] = M[(size_t)i * G + support[c]];
        yy[i] = y[i];
    }
    least_squares(A, m, k, yy, x);
    double ss = 0.0;
    for (int i = 0; i < m; ++i) {
        double s = y[i];
        for (int c = 0; c < k; ++c) s -= M[(size_t)i * G + support[c]] * x[c];
        ss += s * s;
    }
    if (coef) memcpy(coef, x, (size_t)k * sizeof(double));
    if (resid_norm) *resid_norm = sqrt(ss);
    if (margin_out) *margin_out = margin;
    free(r); free(A); free(yy); free(x); free(nrm2); free(taken); free(chosen);
    return 0;
}

/* B sketches y[B][m] against one M: support[B][k], coef[B][k] (or NULL), resid_norm[B] (or NULL), margin[B] (or NULL). */
int cso_block_omp(const double* M, int m, int G, const double* y, int B, int k, int normalised,
                  int32_t* support, double* coef, double* resid_norm, double* margin) {
    int rc = 0;
#pragma omp parallel for schedule(dynamic)
    for (int t = 0; t < B; ++t) {
        const int e = block_omp_one(M, m, G, y + (size_t)t * m, k, normalised, support + (size_t)t * k,
                                    coef ? coef + (size_t)t * k : NULL, resid_norm ? resid_norm + t : NULL, margin ? margin + t : NULL);
        if (e) {
#pragma omp atomic write
            rc = e;
        }
    }
    return rc;
}

/* out[T][d] = sum over g in S_t of Wd_g (silu(Wg_g x_t) * (Wu_g x_t)); Wg, Wu [G][b][d], Wd [G][d][b];
 * support [k] if shared else [T][k]. */
void cso_block_ffn(const double* Wg, const double* Wu, const double* Wd, int G, int b, int d,
                   const double* x, int T, const int32_t* support, int k, int shared, double* out) {
    (void)G;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double* o = out + (size_t)t * d;
        double* h = (double*)malloc((size_t)b * sizeof(double));
        for (int j = 0; j < d; ++j) o[j] = 0.0;
        const int32_t* S = shared ? support : support + (size_t)t * k;
        for (int q = 0; q < k; ++q) {
            const int g = S[q];
            for (int c = 0; c < b; ++c) {
                const double* wg = Wg + ((size_t)g * b + c) * d;
                const double* wu = Wu + ((size_t)g * b + c) * d;
                double gate = 0.0, up = 0.0;
                for (int j = 0; j < d; ++j) { gate += wg[j] * x[(size_t)t * d + j]; up += wu[j] * x[(size_t)t * d + j]; }
                h[c] = gate / (1.0 + exp(-gate)) * up;
            }
            for (int j = 0; j < d; ++j) {
                const double* wd = Wd + ((size_t)g * d + j) * b;
                double s = 0.0;
                for (int c = 0; c < b; ++c) s += wd[c] * h[c];
                o[j] += s;
            }
        }
        free(h);
    }
}

/* out[B][H][dh]: kept heads softmax(q K^T / sqrt(dh)) V over L positions, pruned heads zero.
 * q [B][H][dh]; K, V [B][H][L][dh]; heads [B][kh]. */
void cso_head_attn(const double* q, const double* K, const double* V, int B, int H, int L, int dh,
                   const int32_t* heads, int kh, double* out) {
    for (size_t i = 0; i < (size_t)B * H * dh; ++i) out[i] = 0.0;
#pragma omp parallel for schedule(static)
    for (int item = 0; item < B * kh; ++item) {
        const int bi = item / kh, h = heads[item];
        const double* qv = q + ((size_t)bi * H + h) * dh;
        const double* Kh = K + ((size_t)bi * H + h) * (size_t)L * dh;
        const double* Vh = V + ((size_t)bi * H + h) * (size_t)L * dh;
        double* s = (double*)malloc((size_t)L * sizeof(double));
        double mx = -INFINITY;
        for (int p = 0; p < L; ++p) {
            double v = 0.0;
            for (int j = 0; j < dh; ++j) v += Kh[(size_t)p * dh + j] * qv[j];
            s[p] = v / sqrt((double)dh);
            if (s[p] > mx) mx = s[p];
        }
        double den = 0.0;
        for (int p = 0; p < L; ++p) { s[p] = exp(s[p] - mx); den += s[p]; }
        double* o = out + ((size_t)bi * H + h) * dh;
        for (int j = 0; j < dh; ++j) {
            double v = 0.0;
            for (int p = 0; p < L; ++p) v += s[p] * Vh[(size_t)p * dh + j];
            o[j] = v / den;
        }
        free(s);
    }
}
