// One evaluation of every function sample at the current GP inputs:
//   f_sm(x) = phi_m(x)^T w_sm + k_m(x, X)^T v_sm      and, optionally, d f_sm / d x.
// This is the dominant kernel of a rollout step (Algorithm 1, the sampled transition).
//
// Mapping.  Lane = trajectory.  A wave holds 64 consecutive trajectories and one work unit:
// either CK training points or CL random features of one GP output m.  The operands that
// all trajectories share (scaled training inputs, frequencies) are read through
// wave-uniform addresses, so they travel through the scalar cache into SGPRs and feed the
// vector FMAs as scalar operands; the per-sample streams v and w are read as one float4
// (four consecutive points / features) per lane, coalesced across lanes.  The four waves
// of a workgroup take four consecutive units of the same output and kind for the same 64
// trajectories and add their sums through LDS in wave order; the workgroup writes one
// partial sum [1+D][B] per group of four units, and a later kernel adds the groups up in
// a fixed order, so results do not depend on scheduling.
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
// exp2 takes the integer part and the next eight bits of the exponent from a rounding addition,
// looks 2^(i/256) up in an LDS table and multiplies with a degree-3 polynomial (exp2_tab below).
// Jacobian: d k_mn / d x_d = ln2 * k_mn * (Xs_mnd - log2(e)/l_md^2 x_d); the kernel
// accumulates G_d = sum_n v_n k_n Xs_mnd and u = sum_n v_n k_n, the reduction finishes it.
//
// The random-feature phase is accumulated in float64 in revolutions, reduced exactly to
// [0, 1) and only then rounded to float32 for the hardware sin / cos (which take revolutions).
#include "bagel_internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

// 2^t from u = 256 t.  Adding 1.5 * 2^52 rounds u to the integer J = 256 n + i in the low word of the
// sum (two's complement; |u| < 2^31), so 2^t = 2^n * 2^(i/256) * 2^(g/256) with g = u - J, |g| <= 1/2:
// the middle factor comes from a 256-entry table in LDS (the LDS port is otherwise idle in this
// kernel), the last one from a degree-3 polynomial (relative error 4e-14 over all t), the first one
// from ldexp, which also takes very negative t to zero.  Ten vector instructions; the form without a
// table (degree-7 polynomial for 2^(f/2), squared) takes twelve and is ten times less accurate.
// a3 and a2 come in from the caller, a3 in a scalar and a2 in a vector register: the first Horner
// step is then a single three-operand FMA (an FMA takes at most one scalar operand).
__device__ __forceinline__ double exp2_tab(double u, const double *tab, double a3, double a2)
{
    constexpr double MAGIC = 6755399441055744.0;  // 1.5 * 2^52
    const double s = u + MAGIC;
    const int J = __double2loint(s);
    const double g = u - (s - MAGIC);             // exact
    const double T = tab[J & 255];
    double p = fma(a3, g, a2);
    p = fma(p, g, 0x1.62e42fefa39ddp-9);
    p = fma(p, g, 1.0);
    return ldexp(T * p, J >> 8);
}

// 2^t without a table: split off the integer part, evaluate 2^(f/2) for |f| <= 1/2 with a degree-7
// polynomial and square it (relative error 4e-13), scale with ldexp.  Twelve vector instructions and
// no LDS access.  c7 in a scalar and c6 in a vector register, as in exp2_tab.
__device__ __forceinline__ double exp2_poly(double t, double c7, double c6)
{
    const double n = rint(t);
    const double f = t - n;                       // exact, |f| <= 1/2
    double p = fma(c7, f, c6);
    p = fma(p, f, 4.1667353769980764e-05);
    p = fma(p, f, 0.0006011326659205452);
    p = fma(p, f, 0.006938013583872582);
    p = fma(p, f, 0.060056626759929704);
    p = fma(p, f, 0.3465735902799663);
    p = fma(p, f, 0.9999999999998426);
    return ldexp(p * p, (int)n);
}

// TAB selects the exp2: the table form saves two instructions per training point, but its LDS read
// shares a wait counter with the scalar loads of the shared operands, so every table look-up also
// waits for the operand rows requested ahead.  A launch that fills the chip many times over hides
// that behind other waves (stress workload: 0.647 -> 0.629 ms); a small launch does not (N = 2048,
// B = 1024: 26 -> 35 us), and takes the polynomial form.
template <int D, bool JAC, bool TAB>
__global__ __launch_bounds__(BAGEL_BLOCK) void gp_step_kernel(
    const double *__restrict__ Xs, const double *__restrict__ Os, const double *__restrict__ A,
    const float4 *__restrict__ v4, const float4 *__restrict__ w4, const double *__restrict__ xbuf,
    double *__restrict__ part, const double *__restrict__ exp_tab, int B, int S, int per_sample, int Np, int Lp,
    int CK, int CL, int nck, int ncl, int M)
{
    __shared__ double red[3][1 + D][64];
    __shared__ double tab[256];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b_raw = blockIdx.x * 64 + lane;
    const bool live = b_raw < B;
    const int b = live ? b_raw : B - 1;
    const int sidx = b / per_sample;
    const int group = blockIdx.y;                  // four consecutive units of one output and kind
    const int ngk = (nck + 3) >> 2, ngl = (ncl + 3) >> 2;

    double x[D];
#pragma unroll
    for (int d = 0; d < D; ++d) x[d] = xbuf[(size_t)d * B + b];

    double *out = part + (size_t)group * (1 + D) * B + b;
    double u = 0.0;                                // this wave's sums: value, then the D Jacobian sums
    double G[D];
#pragma unroll
    for (int d = 0; d < D; ++d) G[d] = 0.0;

    if (group < M * ngk) {
        // ---------------- kernel-row unit: CK training points of output m ----------------
        const int m = group / ngk, c = 4 * (group - m * ngk) + wave;
        const int n_iter = c < nck ? CK / 4 : 0;   // a wave past the last chunk adds nothing
        if (TAB) {
            static_assert(BAGEL_BLOCK == 256, "one table entry per thread");
            tab[threadIdx.x] = exp_tab[threadIdx.x];
            __syncthreads();
        }
        double q = 0.0;
#pragma unroll
        for (int d = 0; d < D; ++d) q = fma(-0.5 * A[m * D + d] * x[d], x[d], q);
        // Table form: the exponent is formed times 256 (exact scaling).  exp2_tab needs |256 t| < 2^31:
        // with |q| <= 2^17 and the table rows limited to c_n >= -2^17 (model set-up turns rows beyond
        // that into padding), |t| <= |q| + |c_n| + 2 sqrt(|q| |c_n|) + |log2 alpha^2| < 2^20.  A
        // trajectory further out (about 400 length scales from the origin) is that far from every
        // training point that is kept, and its kernel row is zero: it gets a constant exponent of
        // -3000.  The polynomial form applies the same rule, so both forms agree everywhere.
        const double scale = TAB ? 256.0 : 1.0;
        const bool far = q < -131072.0;
        double xs[D];
#pragma unroll
        for (int d = 0; d < D; ++d) xs[d] = far ? 0.0 : scale * x[d];
        const double qs = far ? -3000.0 * scale : scale * q;
        double kscale = scale;
        const double *__restrict__ Xr = Xs + ((size_t)m * Np + (size_t)c * CK) * (D + 1);
        const float4 *__restrict__ vp = v4 + ((size_t)m * (Np / 4) + (size_t)c * (CK / 4)) * S + sidx;
        // leading polynomial coefficients of the exp2 in use, pinned to register classes (see exp2_tab)
        double ca = TAB ? 0x1.c6b0902a6389dp-29 : 1.192611307487823e-07;
        double cb = TAB ? 0x1.ebfbe3a9ac89ap-19 : 2.409383341728244e-06;
        asm volatile("" : "+s"(ca), "+v"(cb), "+v"(kscale));
        for (int n4 = 0; n4 < n_iter; ++n4) {
            const v4f vv = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(vp + (size_t)n4 * S));   // read-once stream
            const float vj[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double *__restrict__ r = Xr + (size_t)(n4 * 4 + j) * (D + 1);
                double t = TAB ? fma(r[D], kscale, qs) : qs + r[D];
#pragma unroll
                for (int d = 0; d < D; ++d) t = fma(xs[d], r[d], t);
                const double k = TAB ? exp2_tab(t, tab, ca, cb) : exp2_poly(t, ca, cb);
                const double vk = (double)vj[j] * k;
                u += vk;
                if (JAC) {
#pragma unroll
                    for (int d = 0; d < D; ++d) G[d] = fma(vk, r[d], G[d]);
                }
            }
        }
    } else {
        // ---------------- random-feature unit: CL features of output m -------------------
        const int gg = group - M * ngk;
        const int m = gg / ngl, c = 4 * (gg - m * ngl) + wave;
        const int n_iter = c < ncl ? CL / 4 : 0;
        const double *__restrict__ Or = Os + ((size_t)m * Lp + (size_t)c * CL) * (D + 1);
        const float4 *__restrict__ wp = w4 + ((size_t)m * (Lp / 4) + (size_t)c * (CL / 4)) * S + sidx;
        float p = 0.0f;
        for (int l4 = 0; l4 < n_iter; ++l4) {
            const v4f ww = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(wp + (size_t)l4 * S));
            const float wj[4] = {ww.x, ww.y, ww.z, ww.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double *__restrict__ r = Or + (size_t)(l4 * 4 + j) * (D + 1);
                // product first, phase offset last: both are scalar operands, and an FMA takes only one
                double z = x[0] * r[0];
#pragma unroll
                for (int d = 1; d < D; ++d) z = fma(x[d], r[d], z);
                z += r[D];
                // z is the phase in revolutions; its fractional part is exact in float64 and the
                // hardware sin / cos take revolutions (absolute error about one float32 ulp)
                const float y = (float)__builtin_amdgcn_fract(z);
                const float sn = __builtin_amdgcn_sinf(y);
                const float cs = __builtin_amdgcn_cosf(y);
                p = fmaf(wj[j], cs, p);
                if (JAC) {
                    const double ws = (double)(wj[j] * sn);
#pragma unroll
                    for (int d = 0; d < D; ++d) G[d] = fma(ws, r[d], G[d]);
                }
            }
        }
        u = (double)p;
    }

    // waves 1-3 hand their sums to wave 0, which adds them in wave order and writes the group's partial
    if (wave > 0) {
        red[wave - 1][0][lane] = u;
        if (JAC) {
#pragma unroll
            for (int d = 0; d < D; ++d) red[wave - 1][1 + d][lane] = G[d];
        }
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int w = 0; w < 3; ++w) {
            u += red[w][0][lane];
            if (JAC) {
#pragma unroll
                for (int d = 0; d < D; ++d) G[d] += red[w][1 + d][lane];
            }
        }
        if (live) {
            out[0] = u;
            if (JAC) {
#pragma unroll
                for (int d = 0; d < D; ++d) out[(size_t)(1 + d) * B] = G[d];
            }
        }
    }
}

template <int D, bool JAC, bool TAB>
void launch_variant(bagel_ctx *c)
{
    dim3 grid((c->dm.B + 63) / 64, c->groups);
    const int per_sample = c->dm.B / c->dm.S;
    hipLaunchKernelGGL((gp_step_kernel<D, JAC, TAB>), grid, dim3(BAGEL_BLOCK), 0, c->stream, c->Xs, c->Os, c->A, c->v4,
                       c->w4, c->xbuf, c->part, c->exp_tab, c->dm.B, c->dm.S, per_sample, c->Np, c->Lp, c->CK, c->CL,
                       c->nck, c->ncl, c->M);
}

template <int D>
hipError_t launch_d(bagel_ctx *c, bool jac)
{
    if (c->exp_table) {
        if (jac) launch_variant<D, true, true>(c);
        else launch_variant<D, false, true>(c);
    } else {
        if (jac) launch_variant<D, true, false>(c);
        else launch_variant<D, false, false>(c);
    }
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
