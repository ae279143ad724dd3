// Re-layout of the model and of the per-sample streams into the form the step kernel reads.
//   Xs[m][n][0..D-1] = log2(e)/l_md^2 * X_nd,   Xs[m][n][D] = log2(alpha_m^2) - 1/2 sum_d Xs_mnd X_nd
//   Xn[m][n] = the same row with 6144 added to its last entry (rows of the step kernel's table form);
//   near_ok = 0 if a training point or a signal variance lies outside the range of that form
//   Os[m][l][0..D-1] = omega_mld / (2 pi),      Os[m][l][D] = phase_ml / (2 pi)   (revolutions)
//   Of[m][l/4][j][q][l%4] = (float) omega_ml,4q+j / (2 pi), zero for columns >= D: the same frequencies in the
//                           order of the matrix-core operand of the feature Jacobian (see gp_step.hip)
//   v4[m][n/4][s] = v[s][m][4(n/4) .. +3],      w4[m][l/4][s] likewise
// Rows past N (or L) are padding: they evaluate to a kernel value of zero (or a feature of one)
// and carry a zero weight, so they add nothing.  Everything is computed in float64 from the
// float32 inputs (eq. (4) hyper-parameters; random-feature frequencies and phases).
#include "bagel_internal.h"

namespace {

constexpr double LOG2E = 1.4426950408889634074;
constexpr double INV_TWO_PI = 0.15915494309189533577;

__global__ void set_flag_kernel(int *flag, int value) { flag[0] = value; }

__global__ void build_model_kernel(const float *__restrict__ X, const float *__restrict__ ell,
                                   const float *__restrict__ sf2, const float *__restrict__ omega,
                                   const float *__restrict__ phase, double *__restrict__ Xs,
                                   double *__restrict__ Xn, int *__restrict__ near_ok,
                                   double *__restrict__ Os, float *__restrict__ Of, double *__restrict__ A,
                                   double *__restrict__ amp, int M, int N, int L, int D, int Np, int Lp)
{
    const int m = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < Np) {
        double *row = Xs + ((size_t)m * Np + i) * (D + 1);
        if (i < N) {
            double c = log2((double)sf2[m]);
            for (int d = 0; d < D; ++d) {
                const double l = (double)ell[m * D + d];
                const double a = LOG2E / (l * l);
                const double xv = (double)X[(size_t)i * D + d];
                row[d] = a * xv;
                c -= 0.5 * a * xv * xv;
            }
            row[D] = c;
            if (Xn) {
                double *rown = Xn + ((size_t)m * Np + i) * (D + 1);
                for (int d = 0; d < D; ++d) rown[d] = row[d];
                rown[D] = c + 6144.0;
                const double la = log2((double)sf2[m]);
                // the table form needs |c_n| <= 250 and |log2 alpha^2| <= 20 (negated tests: NaN fails them)
                if (!(c >= -250.0) || !(la >= -20.0 && la <= 20.0)) near_ok[0] = 0;
            }
            if (c < -131072.0) {                     // outside the step kernel's range (see gp_step.hip): k = 0
                for (int d = 0; d < D; ++d) row[d] = 0.0;
                row[D] = -2000.0;
            }
        } else {
            for (int d = 0; d < D; ++d) row[d] = 0.0;
            row[D] = -2000.0;
            if (Xn) {                                // padding row of the table form: k = 1, weight 0
                double *rown = Xn + ((size_t)m * Np + i) * (D + 1);
                for (int d = 0; d < D; ++d) rown[d] = 0.0;
                rown[D] = 6144.0;
            }
        }
    }
    if (omega && i < Lp) {
        double *row = Os + ((size_t)m * Lp + i) * (D + 1);
        if (i < L) {
            for (int d = 0; d < D; ++d) row[d] = INV_TWO_PI * (double)omega[((size_t)m * L + i) * D + d];
            row[D] = INV_TWO_PI * (double)phase[(size_t)m * L + i];
        } else {
            for (int d = 0; d <= D; ++d) row[d] = 0.0;
        }
        const int NQ = (D + 3) / 4;
        for (int col = 0; col < 4 * NQ; ++col) {
            const int qd = col >> 2, j = col & 3;
            Of[((((size_t)m * (Lp / 4) + (i >> 2)) * 4 + j) * NQ + qd) * 4 + (i & 3)] = col < D ? (float)row[col] : 0.0f;
        }
    }
    if (i < D) {
        const double l = (double)ell[m * D + i];
        A[m * D + i] = LOG2E / (l * l);
    }
    if (i == 0) amp[m] = sqrt(2.0 * (double)sf2[m] / (double)L);
}

// src[S][M][n] -> dst[M][np/4][S] (float4), zero padded.  One thread per (m, n4, s), s fastest.
__global__ void pack_stream_kernel(const float *__restrict__ src, float4 *__restrict__ dst, int S, int M,
                                   int n, int np4)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)M * np4 * S;
    if (idx >= total) return;
    const int s = (int)(idx % S);
    const size_t r = idx / S;
    const int n4 = (int)(r % np4);
    const int m = (int)(r / np4);
    const float *p = src + ((size_t)s * M + m) * n;
    float t[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int k = n4 * 4 + j;
        t[j] = k < n ? p[k] : 0.0f;
    }
    dst[idx] = make_float4(t[0], t[1], t[2], t[3]);
}

}  // namespace

hipError_t bagel_launch_build_model(bagel_ctx *c, const float *X, const float *ell, const float *sf2,
                                    const float *omega, const float *phase)
{
    const int big = c->Np > c->Lp ? c->Np : c->Lp;
    dim3 grid((big + 255) / 256, c->M);
    // near_ok starts at 1 and is cleared by any row outside the table form's range (contexts without the
    // table form have no Xn)
    if (c->Xn) hipLaunchKernelGGL(set_flag_kernel, dim3(1), dim3(1), 0, c->stream, c->near_ok, 1);
    hipLaunchKernelGGL(build_model_kernel, grid, dim3(256), 0, c->stream, X, ell, sf2, omega, phase, c->Xs, c->Xn,
                       c->near_ok, c->Os, c->Of, c->A, c->amp, c->M, c->dm.N, c->dm.L, c->D, c->Np, c->Lp);
    return hipGetLastError();
}

hipError_t bagel_launch_pack_samples(bagel_ctx *c, const float *w, const float *v)
{
    if (v) {
        const size_t total = (size_t)c->M * (c->Np / 4) * c->dm.S;
        hipLaunchKernelGGL(pack_stream_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, c->stream, v,
                           c->v4, c->dm.S, c->M, c->dm.N, c->Np / 4);
    }
    if (w) {
        const size_t total = (size_t)c->M * (c->Lp / 4) * c->dm.S;
        hipLaunchKernelGGL(pack_stream_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, c->stream, w,
                           c->w4, c->dm.S, c->M, c->dm.L, c->Lp / 4);
    }
    return hipGetLastError();
}
