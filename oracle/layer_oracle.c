/*
 * CPU oracle for one GraphSAGE layer: aggregation followed by the dense update.
 * TEST INFRASTRUCTURE ONLY; shares nothing with the HIP library.
 *
 * What the paper fixes: every layer is the neighbourhood aggregation followed
 * by the MLP operation with one weight matrix per layer (Section 6.3, "Memory
 * and Communication Analysis": w1 is f x h1, w2 is h1 x h2, w3 is h2 x l), and the
 * aggregation is the element-wise sum of the in-neighbours' vectors plus the
 * vertex's own vector, normalised by the in-degree (Section 6.1, "Models and
 * Parameters"), read here as division by din + 1 (see oracle.c, SAGE_GCN).
 *
 *     Z[v, :] = (sum_{u -> v} X[u, :] + X[v, :]) / (din[v] + 1)
 *     H[v, :] = act(Z[v, :] W + b),       act = max(., 0) or identity
 *
 * Readings where the paper is silent: a bias vector and the rectifier as the
 * activation of the hidden layers (the usual GraphSAGE layer); the backward
 * pass is the derivative of the above, with the rectifier's mask taken from
 * the stored forward output (H > 0), as a training framework does.
 *
 * Everything is fp64 scalar loops in the order of the definition.  Next to
 * every result the sum of the absolute values of its terms is accumulated, the
 * scale the rounding-error tolerance of the fp32 GPU path is stated against.
 *
 * Pins (tests/test_oracle_layer_pins.py): numpy's matmul for the dense
 * product (every transpose combination, bias, rectifier), the dense operator
 * (A + I) / (din + 1) for the aggregation, central finite differences of an
 * independent numpy forward for all three gradients, and closed forms.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

/*
 * C[m, n] = act(sum_k opA(A)[m, k] * opB(B)[k, n] + bias[n]).
 * A is stored [M, K] (row stride lda) or, with trans_a, [K, M]; B is stored
 * [K, N] or, with trans_b, [N, K].  C and S are [M, N] fp64, dense.  S (may be
 * NULL) receives sum_k |a * b| + |bias|.
 */
int oracle_matmul(const float *A, int64_t lda, int trans_a, const float *B, int64_t ldb, int trans_b,
                  double *C, double *S, int64_t M, int64_t N, int64_t K, const float *bias, int relu) {
    if (M < 0 || N < 0 || K < 0) return 1;
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0, mag = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double a = trans_a ? (double)A[k * lda + m] : (double)A[m * lda + k];
                double b = trans_b ? (double)B[n * ldb + k] : (double)B[k * ldb + n];
                acc += a * b;
                mag += fabs(a * b);
            }
            if (bias) {
                acc += (double)bias[n];
                mag += fabs((double)bias[n]);
            }
            if (relu && acc < 0.0) acc = 0.0;
            C[m * N + n] = acc;
            if (S) S[m * N + n] = mag;
        }
    }
    return 0;
}

/*
 * Forward of one layer.  X [N, Fi] fp32, W [Fi, Fo] fp32 (row-major), bias [Fo]
 * or NULL.  Outputs (fp64, dense): Z [N, Fi] aggregated input, H [N, Fo], and
 * SH [N, Fo] = sum_k SZ[v, k] |W[k, j]| + |b_j| with SZ the magnitude sum of the
 * aggregation.  Z and SH may be NULL.
 */
int oracle_sage_layer_fwd(const int64_t *indptr, const int32_t *indices, const float *X, const float *W,
                          const float *bias, double *Z, double *H, double *SH,
                          int64_t N, int64_t Fi, int64_t Fo, int relu) {
    double *z = (double *)malloc(sizeof(double) * (size_t)(Fi > 0 ? Fi : 1));
    double *sz = (double *)malloc(sizeof(double) * (size_t)(Fi > 0 ? Fi : 1));
    if (!z || !sz) { free(z); free(sz); return 1; }
    for (int64_t v = 0; v < N; ++v) {
        double din = (double)(indptr[v + 1] - indptr[v]);
        for (int64_t k = 0; k < Fi; ++k) {
            double x = (double)X[v * Fi + k];
            z[k] = x;
            sz[k] = fabs(x);
        }
        for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {
            const float *xu = X + (int64_t)indices[e] * Fi;
            for (int64_t k = 0; k < Fi; ++k) {
                z[k] += (double)xu[k];
                sz[k] += fabs((double)xu[k]);
            }
        }
        for (int64_t k = 0; k < Fi; ++k) {
            z[k] /= din + 1.0;
            sz[k] /= din + 1.0;
            if (Z) Z[v * Fi + k] = z[k];
        }
        for (int64_t j = 0; j < Fo; ++j) {
            double acc = 0.0, mag = 0.0;
            for (int64_t k = 0; k < Fi; ++k) {
                acc += z[k] * (double)W[k * Fo + j];
                mag += sz[k] * fabs((double)W[k * Fo + j]);
            }
            if (bias) {
                acc += (double)bias[j];
                mag += fabs((double)bias[j]);
            }
            if (relu && acc < 0.0) acc = 0.0;
            H[v * Fo + j] = acc;
            if (SH) SH[v * Fo + j] = mag;
        }
    }
    free(z);
    free(sz);
    return 0;
}

/*
 * Backward of one layer.  Inputs: the forward inputs, the stored forward
 * output Hs [N, Fo] fp32 (only its sign is used: the rectifier passes gradient
 * where Hs > 0) and dH [N, Fo] fp32.  With G = dH where the mask allows, else 0:
 *     db[j]    = sum_v G[v, j]
 *     dW[k, j] = sum_v Z[v, k] G[v, j]
 *     dZ[v, k] = sum_j G[v, j] W[k, j]
 *     dX[u, :] = sum_{u -> v} dZ[v, :] / (din[v] + 1)  +  dZ[u, :] / (din[u] + 1)
 * Outputs fp64, dense, each with its magnitude sum (S* may be NULL).
 */
int oracle_sage_layer_bwd(const int64_t *indptr, const int32_t *indices, const float *X, const float *W,
                          const float *Hs, const float *dH, double *dX, double *SdX, double *dW, double *SdW,
                          double *db, double *Sdb, int64_t N, int64_t Fi, int64_t Fo, int relu) {
    size_t nfi = (size_t)(Fi > 0 ? Fi : 1), nfo = (size_t)(Fo > 0 ? Fo : 1);
    double *z = (double *)malloc(sizeof(double) * nfi), *sz = (double *)malloc(sizeof(double) * nfi);
    double *dz = (double *)malloc(sizeof(double) * nfi), *sdz = (double *)malloc(sizeof(double) * nfi);
    double *g = (double *)malloc(sizeof(double) * nfo);
    if (!z || !sz || !dz || !sdz || !g) { free(z); free(sz); free(dz); free(sdz); free(g); return 1; }
    for (int64_t i = 0; i < N * Fi; ++i) { dX[i] = 0.0; if (SdX) SdX[i] = 0.0; }
    for (int64_t i = 0; i < Fi * Fo; ++i) { dW[i] = 0.0; if (SdW) SdW[i] = 0.0; }
    for (int64_t j = 0; j < Fo; ++j) { db[j] = 0.0; if (Sdb) Sdb[j] = 0.0; }
    for (int64_t v = 0; v < N; ++v) {
        double scale = 1.0 / ((double)(indptr[v + 1] - indptr[v]) + 1.0);
        /* aggregated input of this vertex, as in the forward pass */
        for (int64_t k = 0; k < Fi; ++k) { z[k] = (double)X[v * Fi + k]; sz[k] = fabs(z[k]); }
        for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {
            const float *xu = X + (int64_t)indices[e] * Fi;
            for (int64_t k = 0; k < Fi; ++k) { z[k] += (double)xu[k]; sz[k] += fabs((double)xu[k]); }
        }
        for (int64_t k = 0; k < Fi; ++k) { z[k] *= scale; sz[k] *= scale; }
        for (int64_t j = 0; j < Fo; ++j) {
            double pass = (!relu || Hs[v * Fo + j] > 0.0f) ? 1.0 : 0.0;
            g[j] = pass * (double)dH[v * Fo + j];
            db[j] += g[j];
            if (Sdb) Sdb[j] += fabs(g[j]);
        }
        for (int64_t k = 0; k < Fi; ++k) {
            double acc = 0.0, mag = 0.0;
            for (int64_t j = 0; j < Fo; ++j) {
                dW[k * Fo + j] += z[k] * g[j];
                if (SdW) SdW[k * Fo + j] += sz[k] * fabs(g[j]);
                acc += g[j] * (double)W[k * Fo + j];
                mag += fabs(g[j] * (double)W[k * Fo + j]);
            }
            dz[k] = acc * scale;
            sdz[k] = mag * scale;
        }
        /* the adjoint of the aggregation scatters dZ[v] / (din[v] + 1) to v itself and to its in-neighbours */
        for (int64_t k = 0; k < Fi; ++k) {
            dX[v * Fi + k] += dz[k];
            if (SdX) SdX[v * Fi + k] += sdz[k];
        }
        for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {
            int64_t u = indices[e];
            for (int64_t k = 0; k < Fi; ++k) {
                dX[u * Fi + k] += dz[k];
                if (SdX) SdX[u * Fi + k] += sdz[k];
            }
        }
    }
    free(z); free(sz); free(dz); free(sdz); free(g);
    return 0;
}
