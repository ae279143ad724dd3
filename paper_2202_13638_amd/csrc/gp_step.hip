// One evaluation of every function sample at the current GP inputs:
//   f_sm(x) = phi_m(x)^T w_sm + k_m(x, X)^T v_sm      and, optionally, d f_sm / d x.
// This is the dominant kernel of a rollout step (Algorithm 1, the sampled transition).
//
// Mapping.  Lane = trajectory.  A workgroup holds 256 consecutive trajectories and one
// work unit: either CK training points or CL random features of one GP output m.  The
// operands that all trajectories share (scaled training inputs, frequencies) are read
// through wave-uniform addresses, so they travel through the scalar cache into SGPRs and
// feed the vector FMAs as scalar operands; the per-sample streams v and w are read as
// one float4 (four consecutive points / features) per lane, coalesced across lanes.
// Each unit writes its partial sums [1+D][B]; a later kernel adds the units up in a fixed
// order, so results do not depend on scheduling.
//
// Arithmetic.  The kernel row is evaluated in float64: with noise variance far below the
// signal variance the representer weights v are large with alternating signs, the sum
// cancels by many orders of magnitude, and float32 rounding of each exp() alone would
// exceed the error budget of a rollout.  gfx950 issues float64 FMAs at the same rate as
// unpacked float32 FMAs, so this costs registers, not throughput.  In float64 the squared
// distance can be expanded, which turns  -1/2 |x - X_n|^2_Lambda  into one dot product
// against pre-scaled inputs plus two precomputed terms:
//   log2 k_mn(x) = q_m(x) + c_mn + sum_d x_d * Xs_mnd,
//   Xs_mnd = log2(e)/l_md^2 * X_nd,  c_mn = log2(alpha_m^2) - 1/2 sum_d Xs_mnd X_nd,
//   q_m(x) = -1/2 sum_d log2(e)/l_md^2 x_d^2.
// exp2 is a degree-10 polynomial on [-1/2, 1/2] after splitting off the integer part.
// Jacobian: d k_mn / d x_d = ln2 * k_mn * (Xs_mnd - log2(e)/l_md^2 x_d); the kernel
// accumulates G_d = sum_n v_n k_n Xs_mnd and u = sum_n v_n k_n, the reduction finishes it.
//
// The random-feature phase is accumulated in float64 in quarter revolutions, reduced
// exactly to [-1/2, 1/2] and only then rounded to float32 for a polynomial sin/cos.
#include "bagel_internal.h"

namespace {

__device__ __forceinline__ double exp2_poly(double t)
{
    // t <= log2(alpha^2); clamp the far tail so the integer part stays representable
    t = fmax(t, -1040.0);
    const double n = rint(t);
    const double f = t - n;                       // exact, |f| <= 1/2
    double p = 6.767963482574983e-09;
    p = fma(p, f, 1.0206977921453389e-07);
    p = fma(p, f, 1.3217210256367588e-06);
    p = fma(p, f, 1.525266622014565e-05);
    p = fma(p, f, 0.00015403526882354606);
    p = fma(p, f, 0.0013333558214738293);
    p = fma(p, f, 0.00961812911053657);
    p = fma(p, f, 0.055504108664544756);
    p = fma(p, f, 0.24022650695901254);
    p = fma(p, f, 0.6931471805599483);
    p = fma(p, f, 1.0);
    return ldexp(p, (int)n);
}

// sin and cos of (pi/2) * (j + y), j integer, |y| <= 1/2
__device__ __forceinline__ void sincos_quarter(float y, int j, float &sn, float &cs)
{
    const float u = y * y;
    float s = -0.004602149212814766f;
    s = fmaf(s, u, 0.07968021764776267f);
    s = fmaf(s, u, -0.6459634776648127f);
    s = fmaf(s, u, 1.5707963219532366f);
    s *= y;
    float c = 0.0009036280586426939f;
    c = fmaf(c, u, -0.02086006949632079f);
    c = fmaf(c, u, 0.25366920365446266f);
    c = fmaf(c, u, -1.2337005406331254f);
    c = fmaf(c, u, 1.0f);
    // rotate by j quarter turns
    const bool swap = (j & 1) != 0;
    float a = swap ? c : s;       // |sin|
    float b = swap ? s : c;       // |cos|
    // sin((pi/2)(j+y)): j=0: s, 1: c, 2: -s, 3: -c ; cos: j=0: c, 1: -s, 2: -c, 3: s
    sn = (j & 2) ? -a : a;
    cs = ((j + 1) & 2) ? -b : b;
}

template <int D, bool JAC>
__global__ __launch_bounds__(BAGEL_BLOCK) void gp_step_kernel(
    const double *__restrict__ Xs, const double *__restrict__ Os, const double *__restrict__ A,
    const float4 *__restrict__ v4, const float4 *__restrict__ w4, const double *__restrict__ xbuf,
    double *__restrict__ part, int B, int S, int per_sample, int Np, int Lp, int CK, int CL, int nck,
    int ncl, int M)
{
    const int b_raw = blockIdx.x * BAGEL_BLOCK + threadIdx.x;
    const bool live = b_raw < B;
    const int b = live ? b_raw : B - 1;
    const int sidx = b / per_sample;
    const int unit = blockIdx.y;

    double x[D];
#pragma unroll
    for (int d = 0; d < D; ++d) x[d] = xbuf[(size_t)d * B + b];

    double *out = part + (size_t)unit * (1 + D) * B + b;

    if (unit < M * nck) {
        // ---------------- kernel-row unit: CK training points of output m ----------------
        const int m = unit / nck, c = unit - m * nck;
        double q = 0.0;
#pragma unroll
        for (int d = 0; d < D; ++d) q = fma(-0.5 * A[m * D + d] * x[d], x[d], q);
        const double *__restrict__ Xr = Xs + ((size_t)m * Np + (size_t)c * CK) * (D + 1);
        const float4 *__restrict__ vp = v4 + ((size_t)m * (Np / 4) + (size_t)c * (CK / 4)) * S + sidx;
        double u = 0.0;
        double G[D];
#pragma unroll
        for (int d = 0; d < D; ++d) G[d] = 0.0;
        for (int n4 = 0; n4 < CK / 4; ++n4) {
            const float4 vv = vp[(size_t)n4 * S];
            const float vj[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double *__restrict__ r = Xr + (size_t)(n4 * 4 + j) * (D + 1);
                double t = q + r[D];
#pragma unroll
                for (int d = 0; d < D; ++d) t = fma(x[d], r[d], t);
                const double k = exp2_poly(t);
                const double vk = (double)vj[j] * k;
                u += vk;
                if (JAC) {
#pragma unroll
                    for (int d = 0; d < D; ++d) G[d] = fma(vk, r[d], G[d]);
                }
            }
        }
        if (live) {
            out[0] = u;
            if (JAC) {
#pragma unroll
                for (int d = 0; d < D; ++d) out[(size_t)(1 + d) * B] = G[d];
            }
        }
    } else {
        // ---------------- random-feature unit: CL features of output m -------------------
        const int uu = unit - M * nck;
        const int m = uu / ncl, c = uu - m * ncl;
        const double *__restrict__ Or = Os + ((size_t)m * Lp + (size_t)c * CL) * (D + 1);
        const float4 *__restrict__ wp = w4 + ((size_t)m * (Lp / 4) + (size_t)c * (CL / 4)) * S + sidx;
        float p = 0.0f;
        double G[D];
#pragma unroll
        for (int d = 0; d < D; ++d) G[d] = 0.0;
        for (int l4 = 0; l4 < CL / 4; ++l4) {
            const float4 ww = wp[(size_t)l4 * S];
            const float wj[4] = {ww.x, ww.y, ww.z, ww.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double *__restrict__ r = Or + (size_t)(l4 * 4 + j) * (D + 1);
                double z = r[D];
#pragma unroll
                for (int d = 0; d < D; ++d) z = fma(x[d], r[d], z);
                const double zi = rint(z);
                const float y = (float)(z - zi);
                // the quadrant only matters modulo 4; reduce in float64 before converting
                const int jq = (int)(zi - 4.0 * floor(zi * 0.25));
                float sn, cs;
                sincos_quarter(y, jq, sn, cs);
                p = fmaf(wj[j], cs, p);
                if (JAC) {
                    const double ws = (double)(wj[j] * sn);
#pragma unroll
                    for (int d = 0; d < D; ++d) G[d] = fma(ws, r[d], G[d]);
                }
            }
        }
        if (live) {
            out[0] = (double)p;
            if (JAC) {
#pragma unroll
                for (int d = 0; d < D; ++d) out[(size_t)(1 + d) * B] = G[d];
            }
        }
    }
}

template <int D>
hipError_t launch_d(bagel_ctx *c, bool jac)
{
    dim3 grid((c->dm.B + BAGEL_BLOCK - 1) / BAGEL_BLOCK, c->units);
    const int per_sample = c->dm.B / c->dm.S;
    if (jac)
        hipLaunchKernelGGL((gp_step_kernel<D, true>), grid, dim3(BAGEL_BLOCK), 0, c->stream, c->Xs, c->Os, c->A,
                           c->v4, c->w4, c->xbuf, c->part, c->dm.B, c->dm.S, per_sample, c->Np, c->Lp, c->CK,
                           c->CL, c->nck, c->ncl, c->M);
    else
        hipLaunchKernelGGL((gp_step_kernel<D, false>), grid, dim3(BAGEL_BLOCK), 0, c->stream, c->Xs, c->Os, c->A,
                           c->v4, c->w4, c->xbuf, c->part, c->dm.B, c->dm.S, per_sample, c->Np, c->Lp, c->CK,
                           c->CL, c->nck, c->ncl, c->M);
    return hipGetLastError();
}

}  // namespace

hipError_t bagel_launch_gp_step(bagel_ctx *c, bool jac)
{
    switch (c->D) {
#define CASE(n) case n: return launch_d<n>(c, jac);
        CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12)
        CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
    }
    return hipErrorInvalidValue;
}
