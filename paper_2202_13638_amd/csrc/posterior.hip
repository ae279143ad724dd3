// Per-step posterior sampler: Algorithm 1 as printed draws the next state at every step from the
// predictive posterior of the GPs (eq. (9)), one independent GP per state increment (Sec. III-A):
//   f_m = mu_m(x) + sqrt(var_m(x)) xi_m,    xi ~ N(0, 1) supplied by the caller (reparameterised draw),
//   mu_m(x)  = k_m(x, X)^T alpha_m,                  alpha_m = K_hat_m^-1 y_m          (eq. (2), zero prior mean)
//   var_m(x) = alpha_m^2 - k_m(x, X)^T K_hat_m^-1 k_m(x, X)                             (eq. (3))
// with the exact K_hat^-1 from bagel_prepare_posterior (the paper speeds the variance up with Lanczos
// estimates of the same quantity; that approximation is not reproduced here).
//
// One step, per output m, for all B trajectories at once:
//   1. posterior_rows_kernel: Kx[n][b] = k_m(x_b, X_n) in float64 (lane = trajectory, training inputs as
//      scalar operands, the same expanded-distance form and software exp2 as the pathwise step kernel);
//   2. Q = K_hat_m^-1 Kx: one float64 GEMM [Np x Np] x [Np x B], the dominant cost (2 N^2 flop per
//      trajectory, step and output);
//   3. posterior_reduce_kernel: mu, var and their derivatives from Kx, Q, alpha and the scaled inputs,
//        d mu / d x_d  = ln2 (sum_n alpha_n k_n Xs_nd - A_d x_d sum_n alpha_n k_n),
//        d var / d x_d = -2 ln2 (sum_n q_n k_n Xs_nd - A_d x_d sum_n q_n k_n),
//      then f and J = d mu + xi / (2 sqrt(var)) d var, written in the layout the end-of-step kernel reads.
// A variance below 1e-12 is held there and its derivative set to zero.
// Everything after that (state update, cost, tape, policy, backward sweep) is shared with the pathwise sampler.
#include "bagel_internal.h"

namespace {

constexpr double LN2 = 0.69314718055994530942;
constexpr double VAR_FLOOR = 1e-12;

__device__ __forceinline__ double exp2_f64(double t)
{
    const double n = rint(t);
    const double f = t - n;                       // exact, |f| <= 1/2
    double p = 1.192611307487823e-07;             // degree-7 polynomial for 2^(f/2), squared below
    p = fma(p, f, 2.409383341728244e-06);
    p = fma(p, f, 4.1667353769980764e-05);
    p = fma(p, f, 0.0006011326659205452);
    p = fma(p, f, 0.006938013583872582);
    p = fma(p, f, 0.060056626759929704);
    p = fma(p, f, 0.3465735902799663);
    p = fma(p, f, 0.9999999999998426);
    return ldexp(p * p, (int)n);
}

// Kx[n][b] for n in [32 blockIdx.y, +32), b = lane; rows n >= N (padding) are zero
template <int D>
__global__ __launch_bounds__(256) void posterior_rows_kernel(const double *__restrict__ Xs_m, const double *__restrict__ A_m,
                                                             const double *__restrict__ xbuf, double *__restrict__ Kx,
                                                             int B, int N, int Np)
{
    const int b_raw = blockIdx.x * 256 + threadIdx.x;
    const bool live = b_raw < B;
    const int b = live ? b_raw : B - 1;
    double x[D];
#pragma unroll
    for (int d = 0; d < D; ++d) x[d] = xbuf[(size_t)d * B + b];
    double q = 0.0;
#pragma unroll
    for (int d = 0; d < D; ++d) q = fma(-0.5 * A_m[d] * x[d], x[d], q);
    const int n0 = blockIdx.y * 32;
    for (int n = n0; n < n0 + 32 && n < Np; ++n) {
        double k = 0.0;
        if (n < N) {
            const double *__restrict__ r = Xs_m + (size_t)n * (D + 1);
            double t = q + r[D];
#pragma unroll
            for (int d = 0; d < D; ++d) t = fma(x[d], r[d], t);
            k = exp2_f64(t);
        }
        if (live) Kx[(size_t)n * B + b] = k;
    }
}

// Workgroup = 64 trajectories x 16 slices of the training points, one component (comp 0 -> f,
// comp 1 + d -> J[d]) per blockIdx.y; the slices' sums are added through LDS in slice order, then
// slice 0 finishes the moments.  out[comp * B + b] of output m.
template <int D>
__global__ __launch_bounds__(1024) void posterior_reduce_kernel(const double *__restrict__ Xs_m, const double *__restrict__ A_m,
                                                                const double *__restrict__ alpha_m,
                                                                const double *__restrict__ Kx, const double *__restrict__ Q,
                                                                const double *__restrict__ xbuf,
                                                                const float *__restrict__ xi_t, double sf2,
                                                                double *__restrict__ out, int B, int N, int M, int m)
{
    __shared__ double red[15][4][64];
    const int lane = threadIdx.x & 63;
    const int slice = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b_raw = blockIdx.x * 64 + lane;
    const bool live = b_raw < B;
    const int b = live ? b_raw : B - 1;
    const int comp = blockIdx.y;
    const int d = comp - 1;
    const int per = (N + 15) / 16;
    const int n_begin = slice * per, n_end = min(N, n_begin + per);
    double mu = 0.0, quad = 0.0, gmu = 0.0, gq = 0.0;
    for (int n = n_begin; n < n_end; ++n) {
        const double k = Kx[(size_t)n * B + b];
        const double ak = alpha_m[n] * k, qk = Q[(size_t)n * B + b] * k;
        mu += ak;
        quad += qk;
        if (comp > 0) {
            const double xs = Xs_m[(size_t)n * (D + 1) + d];
            gmu = fma(ak, xs, gmu);
            gq = fma(qk, xs, gq);
        }
    }
    if (slice > 0) {
        red[slice - 1][0][lane] = mu; red[slice - 1][1][lane] = quad;
        red[slice - 1][2][lane] = gmu; red[slice - 1][3][lane] = gq;
    }
    __syncthreads();
    if (slice > 0 || !live) return;
    for (int s = 0; s < 15; ++s) {
        mu += red[s][0][lane]; quad += red[s][1][lane]; gmu += red[s][2][lane]; gq += red[s][3][lane];
    }
    double var = sf2 - quad;
    const bool floored = var < VAR_FLOOR;
    if (floored) var = VAR_FLOOR;
    const double sd = sqrt(var);
    const double z = (double)xi_t[(size_t)b * M + m];
    if (comp == 0) {
        out[b] = mu + sd * z;
    } else {
        const double ax = A_m[d] * xbuf[(size_t)d * B + b];
        const double dmu = LN2 * (gmu - ax * mu);
        const double dvar = floored ? 0.0 : -2.0 * LN2 * (gq - ax * quad);
        out[(size_t)comp * B + b] = dmu + z * dvar / (2.0 * sd);
    }
}

template <int D>
hipError_t step_d(bagel_ctx *c, bool jac, const float *xi_t)
{
    const int B = c->dm.B, N = c->dm.N, Np = c->post_Np, M = c->M;
    for (int m = 0; m < M; ++m) {
        const double *Xs_m = c->Xs + (size_t)m * c->Np * (D + 1);
        const double *A_m = c->A + (size_t)m * D;
        hipLaunchKernelGGL((posterior_rows_kernel<D>), dim3((B + 255) / 256, (Np + 31) / 32), dim3(256), 0, c->stream, Xs_m,
                           A_m, c->xbuf, c->post_Kx, B, N, Np);
        bagel_dgemm(c->stream, Np, B, Np, 1.0, c->post_Kinv + (size_t)m * Np * Np, Np, 1, c->post_Kx, B, 1, c->post_Q, B, true);
        hipLaunchKernelGGL((posterior_reduce_kernel<D>), dim3((B + 63) / 64, jac ? 1 + D : 1), dim3(1024), 0, c->stream,
                           Xs_m, A_m, c->post_alpha + (size_t)m * Np, c->post_Kx, c->post_Q, c->xbuf, xi_t, c->post_sf2[m],
                           c->part + (size_t)m * (1 + D) * B, B, N, M, m);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t bagel_launch_posterior_step(bagel_ctx *c, bool jac, const float *xi_t)
{
    switch (c->D) {
#define CASE(n) case n: return step_d<n>(c, jac, xi_t);
        CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12)
        CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
    }
    return hipErrorInvalidValue;
}
