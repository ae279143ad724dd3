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
// exp2 is evaluated in software (there is no float64 exp instruction): a polynomial form for any
// argument (exp2_poly), and a table form for the normal range that reads the split of the exponent
// straight off the bits of a sum (see gp_step_kernel).
// Jacobian: d k_mn / d x_d = ln2 * k_mn * (Xs_mnd - log2(e)/l_md^2 x_d); the kernel
// accumulates G_d = sum_n v_n k_n Xs_mnd and u = sum_n v_n k_n, the reduction finishes it.
//
// The random-feature phase is accumulated in float64 in revolutions, reduced exactly to
// [0, 1) and only then rounded to float32 for the hardware sin / cos (which take revolutions).
#include <stdlib.h>

#include "bagel_internal.h"

namespace {

#ifndef BAGEL_MIN_WAVES
#define BAGEL_MIN_WAVES(D) ((D) <= 8 ? 8 : ((D) <= 11 ? 5 : 4))
#endif
#ifndef BAGEL_SAME_ROWS
#define BAGEL_SAME_ROWS 0      // timing experiment only: every work unit reads the first unit's rows
#endif

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float f4v __attribute__((ext_vector_type(4)));

// The per-sample streams (v and w) are read through buffer loads: a wave-uniform descriptor of the
// work unit's rows, a wave-uniform row offset that the scalar unit advances, and a constant 32-bit
// byte offset per lane (the lane's sample).  The load instruction adds the three itself, so the loop
// spends no vector instruction on addresses.  Non-temporal: each float4 is read once per launch.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t stream_descriptor(const float4 *rows, size_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float4 *>(rows), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ v4f stream_load(__amdgpu_buffer_rsrc_t desc, unsigned lane_off, unsigned row_off)
{
    return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(desc, lane_off, row_off, 2));
}

// 2^t without a table: split off the integer part, evaluate 2^(f/2) for |f| <= 1/2 with a degree-7
// polynomial and square it (relative error 4e-13), scale with ldexp.  Twelve vector instructions and
// no LDS access.  c7 comes in a scalar and c6 in a vector register: the first Horner step is then a
// single three-operand FMA (an FMA takes at most one scalar operand).
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

// End of a workgroup: waves 1-3 hand their sums (value u, Jacobian sums G) to wave 0 through LDS slots
// 0-2, wave 0 adds them in wave order and writes the group's partial sum.  in_lds: every wave, wave 0
// included (slot 3), has already stored its sums (the feature units of a Jacobian launch).
template <int D, bool JAC, int RC>
__device__ __forceinline__ void combine_waves(double (*red)[RC][64], int wave, int lane, bool live, double *out, int B,
                                              bool in_lds, double u, double (&G)[D])
{
    if (wave > 0 && !in_lds) {
        red[wave - 1][0][lane] = u;
        if (JAC) {
#pragma unroll
            for (int d = 0; d < D; ++d) red[wave - 1][1 + d][lane] = G[d];
        }
    }
    __syncthreads();
    if (wave == 0) {
        if (in_lds) {
            u = red[3][0][lane];
#pragma unroll
            for (int d = 0; d < D; ++d) G[d] = red[3][1 + d][lane];
        }
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

// ---- Jacobian sums of one step, added up --------------------------------------------------------
// J[m][d] = -amp_m (2 pi) sum_g Gr_g[d] + ln2 (sum_g Gk_g[d] - log2(e)/l_md^2 x_d sum_g u_g)   (groups in order)
// for the 64 trajectories of one tile, from the partial sums `part` of a sample evaluation at x; the
// result goes to a slot of the Jacobian tape, jdst[M][D][B] (float32).  Nothing on the critical path of
// a rollout needs J, so this runs as M extra rows of workgroups (one per output) inside the NEXT step's
// sample evaluation (or, after the last step, as a launch of its own).  256 threads: the four waves
// share the D entries of the output.
struct jac_sums {
    const double *part;      // [groups][1+D][B]
    const double *x;         // [D][B] inputs the sums were evaluated at
    const double *A, *amp;   // [M][D], [M]
    float *jdst;             // [M][D][B]
};

__device__ __forceinline__ double sum_in_order(const double *__restrict__ p, int n, size_t stride)
{
    double s = 0.0;
    for (int c0 = 0; c0 < n; c0 += 4) {      // four loads in flight at a time, added in order
        double v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = (c0 + i < n) ? p[(size_t)(c0 + i) * stride] : 0.0;
#pragma unroll
        for (int i = 0; i < 4; ++i) s += v[i];
    }
    return s;
}

__device__ __forceinline__ void jacobian_tile(const jac_sums &j, int tile, int m, int B, int D, int M, int ngk, int ngl)
{
    constexpr double LN2 = 0.69314718055994530942, TWO_PI = 6.28318530717958647693;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = tile * 64 + lane;
    if (b >= B) return;
    const size_t stride = (size_t)(1 + D) * B;
    const double *pk = j.part + (size_t)(m * ngk) * stride + b;
    const double *pr = j.part + (size_t)(M * ngk + m * ngl) * stride + b;
    const double u = sum_in_order(pk, ngk, stride);
    for (int d = wave; d < D; d += BAGEL_BLOCK / 64) {
        const double gk = sum_in_order(pk + (size_t)(1 + d) * B, ngk, stride);
        const double gr = sum_in_order(pr + (size_t)(1 + d) * B, ngl, stride);
        const double xd = j.x[(size_t)d * B + b];
        j.jdst[(size_t)(m * D + d) * B + b] = (float)(-j.amp[m] * TWO_PI * gr + LN2 * (gk - j.A[m * D + d] * xd * u));
    }
}

__global__ __launch_bounds__(BAGEL_BLOCK) void jac_reduce_kernel(jac_sums j, int B, int D, int M, int ngk, int ngl)
{
    jacobian_tile(j, blockIdx.x, blockIdx.y, B, D, M, ngk, ngl);
}

// NEAR adds the fast form of the kernel-row loop for the normal case that data and trajectory are
// within about 19 length scales of the origin; the loop above is then the fallback of a wave that
// holds a trajectory further out, or of a model with training points further out (near_ok == 0).
// With  q = -1/2 sum_d a_d x_d^2  taken out of the exponent (the sums are multiplied by 2^q at the end),
//   t'_n = c_n + sum_d x_d Xs_nd   lies in [-770, 270]   for |q|, |c_n| <= 250 and |log2 alpha^2| <= 20,
// and the near table holds c_n + 6144 in place of c_n: 6144 = 1.5 * 2^12 puts the sum s = t'_n + 6144 into
// [2^12, 2^13), where one unit in the last place is 2^-40, so the bits of s ARE the split of t'_n:
//   high word bits 19..8 = 2048 + floor(t'), bits 7..0 = the next eight bits i (t' in units of 1/256),
//   low word = the remaining fraction g in units of 2^-40 (t' rounded to 2^-41: relative error 3e-13 of k).
// Then 2^t' = 2^floor(t') * 2^(i/256) * 2^g: the middle factor comes from a 256-entry table in LDS,
// indexed by the low byte of the high word; 2^g is a degree-3 polynomial in the low word converted to
// float64 (coefficients pre-scaled by 2^-40k; relative error 7e-14 on [0, 2^-8)); and the power of two is
// applied by adding the high word of s, shifted left by 12, to the high word of the table entry: the
// shift drops the exponent of s and leaves (2048 + floor t') << 20 | i << 12, so the table stores
// 2^(i/256) with i << 12 subtracted from its high word and its sign bit set (adding 2048 << 20 clears
// it again).  No exponent can wrap for t' in the range above.  Per training point: 9 instructions for s,
// 7 for k (address, conversion, 3 polynomial steps, exponent add, product), 2 for v k, 9 to accumulate
// = 27, against 32 of the general loop.
// The table form needs many workgroups per compute unit to pay: its LDS read shares a wait counter
// with the scalar loads of the shared operands, so every look-up also waits for the operand rows
// requested ahead; small launches take the general loop only.
template <int D, bool JAC, bool NEAR>
__global__ __launch_bounds__(BAGEL_BLOCK) __attribute__((amdgpu_waves_per_eu(BAGEL_MIN_WAVES(D), 8))) void gp_step_kernel(
    const double *__restrict__ Xs, const double *__restrict__ Xn, const double *__restrict__ Os,
    const float4 *__restrict__ Of, const double *__restrict__ A, const float4 *__restrict__ v4,
    const float4 *__restrict__ w4,
    const double *__restrict__ xbuf, double *__restrict__ part, const double *__restrict__ exp_tab,
    const int *__restrict__ near_ok, int B, int S, int per_sample, int Np, int Lp, int CK, int CL, int nck, int ncl,
    int M, jac_sums prev)
{
    // M rows of workgroups past the work units: the previous step's Jacobian sums (see jacobian_tile).
    // (Placed first in the grid instead, they made the launch slower: 571 vs 556 us.)
    if ((int)blockIdx.y >= M * (((nck + 3) >> 2) + ((ncl + 3) >> 2))) {
        jacobian_tile(prev, blockIdx.x, (int)blockIdx.y - M * (((nck + 3) >> 2) + ((ncl + 3) >> 2)), B, D, M,
                      (nck + 3) >> 2, (ncl + 3) >> 2);
        return;
    }
    // Sums handed from wave to wave at the end.  Slot 3 is used only by the feature units of a
    // Jacobian launch; the kernel-row units keep the table of the table form there.
    constexpr int RC = 1 + D > 4 ? 1 + D : 4;      // rows per slot: at least the 256 entries of the exp2 table
    __shared__ double red[4][RC][64];
    double *tab = &red[3][0][0];
    constexpr int NQ = (D + 3) / 4;                // matrix instructions per feature: four Jacobian columns each
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

    if (group < M * ngk) {
        double u = 0.0;                            // this wave's sums: value, then the D Jacobian sums
        double G[D];
#pragma unroll
        for (int d = 0; d < D; ++d) G[d] = 0.0;
        // ---------------- kernel-row unit: CK training points of output m ----------------
        const int m = group / ngk, c = 4 * (group - m * ngk) + wave;
        const int n_iter = c < nck ? CK / 4 : 0;   // a wave past the last chunk adds nothing
        if (NEAR) {
            static_assert(BAGEL_BLOCK == 256, "one table entry per thread");
            tab[threadIdx.x] = exp_tab[threadIdx.x];
            __syncthreads();
        }
        double q = 0.0;
#pragma unroll
        for (int d = 0; d < D; ++d) q = fma(-0.5 * A[m * D + d] * x[d], x[d], q);
        const size_t row0 = BAGEL_SAME_ROWS ? 0 : ((size_t)m * Np + (size_t)c * CK) * (D + 1);
        // the stream of this unit for this lane's sample: uniform base address plus a 32-bit lane offset
        const unsigned vstep = (unsigned)S * (unsigned)sizeof(float4);       // one row: four points of every sample
        const float4 *vrows = v4 + ((size_t)m * (Np / 4) + (size_t)c * (CK / 4)) * S;
        const unsigned voff = (unsigned)sidx * (unsigned)sizeof(float4);
        bool wave_near = false;
        if (NEAR) wave_near = near_ok[0] != 0 && !__any(!(q >= -250.0));
        // (Each of the two loops builds the stream's descriptor for itself, from a base pointer the
        // compiler cannot identify with the other loop's: one shared descriptor would live across both
        // loops, and the scalar-register pressure of the general loop would then spill it inside the
        // table loop too - eleven extra vector instructions per eight points.)
        if (NEAR && wave_near) {
            const float4 *vrows_t = vrows;
            asm volatile("" : "+s"(vrows_t));
            const __amdgpu_buffer_rsrc_t vdesc = stream_descriptor(vrows_t, (size_t)(CK / 4) * vstep);
            const double *__restrict__ Xr = Xn + row0;
            const int last = n_iter - 1;
            // leading polynomial coefficients pinned to register classes: the first Horner step is then a
            // single three-operand FMA (an FMA takes at most one scalar operand)
            double ca = 0x1.c726cfe5bfc26p-125, cb = 0x1.ebfbd4e173a43p-83;
            asm volatile("" : "+s"(ca), "+v"(cb));
            {
                // One training point with its row in rc; the next point's row is requested into rn right at
                // the start, so that its trip through the scalar cache overlaps this point's arithmetic and
                // table look-up instead of preceding the next point's.
                auto one_point = [&](const double (&rc)[D + 1], double (&rn)[D + 1], const double *__restrict__ next,
                                     float vf) {
#pragma unroll
                    for (int d = 0; d <= D; ++d) rn[d] = next[d];
                    __builtin_amdgcn_sched_barrier(0);
                    double t = x[0] * rc[0];
#pragma unroll
                    for (int d = 1; d < D; ++d) t = fma(x[d], rc[d], t);
                    const double s = t + rc[D];
                    const int hs = __double2hiint(s);
                    const double T = tab[hs & 255];
                    const double g = (double)(unsigned)__double2loint(s);
                    double p = fma(ca, g, cb);
                    p = fma(p, g, 0x1.62e42fefcb0c8p-41);
                    p = fma(p, g, 1.0);
                    const double sc = __hiloint2double(__double2hiint(T) + (hs << 12), __double2loint(T));
                    const double vk = (double)vf * (sc * p);
                    u += vk;
                    if (JAC) {
#pragma unroll
                        for (int d = 0; d < D; ++d) G[d] = fma(vk, rc[d], G[d]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                };
                double ra[D + 1], rb[D + 1];
#pragma unroll
                for (int d = 0; d <= D; ++d) ra[d] = Xr[d];
                // rows follow each other in memory; the request past the unit's last row reads the first
                // row of the next unit or, after the very last one, stays inside the table (see below)
                auto four_points = [&](const v4f vv, int n4) {
                    const double *__restrict__ r = Xr + (size_t)(n4 * 4) * (D + 1);
                    one_point(ra, rb, r + 1 * (D + 1), vv.x);
                    one_point(rb, ra, r + 2 * (D + 1), vv.y);
                    one_point(ra, rb, r + 3 * (D + 1), vv.z);
                    one_point(rb, ra, n4 < last ? r + 4 * (D + 1) : Xr, vv.w);
                };
                // The stream is requested one float4 ahead, alternating between two register sets (a request
                // past the end repeats the last row): HBM latency under load is several times a wave's own
                // work on four points, and the loop was idle waiting for it.
                // (CK is a multiple of 8: the loop body handles two float4 without a branch, which keeps
                // the compiler from moving a request down to its use.)
                v4f va = stream_load(vdesc, voff, 0u);
                for (int n4 = 0; n4 < n_iter; n4 += 2) {
                    const v4f vb = stream_load(vdesc, voff, (unsigned)(n4 + 1) * vstep);
                    four_points(va, n4);
                    va = stream_load(vdesc, voff, (unsigned)(n4 + 2 < last ? n4 + 2 : last) * vstep);
                    four_points(vb, n4 + 1);
                }
            }
            // 2^q (q in [-250, 0]) by the loop's own table form: it needs no constants beyond the loop's,
            // whereas the polynomial form's seven would be kept in scalar registers across the loop
            // (shared with the general loop below) and push the loop's operands out into spill lanes
            const double sq = q + 6144.0;
            const int hq = __double2hiint(sq);
            const double Tq = tab[hq & 255];
            const double gq = (double)(unsigned)__double2loint(sq);
            double pq = fma(ca, gq, cb);
            pq = fma(pq, gq, 0x1.62e42fefcb0c8p-41);
            pq = fma(pq, gq, 1.0);
            const double eq = pq * __hiloint2double(__double2hiint(Tq) + (hq << 12), __double2loint(Tq));
            u *= eq;
            if (JAC) {
#pragma unroll
                for (int d = 0; d < D; ++d) G[d] *= eq;
            }
        } else {
            // A trajectory further out than about 400 length scales (q < -2^17) is that far from every
            // training point that is kept (model set-up turns rows with c_n < -2^17 into padding), and its
            // kernel row is zero: it gets a constant exponent of -3000.
            const float4 *vrows_g = vrows;
            asm volatile("" : "+s"(vrows_g));
            const __amdgpu_buffer_rsrc_t vdesc = stream_descriptor(vrows_g, (size_t)(CK / 4) * vstep);
            const bool far = q < -131072.0;
            double xs[D];
#pragma unroll
            for (int d = 0; d < D; ++d) xs[d] = far ? 0.0 : x[d];
            const double qs = far ? -3000.0 : q;
            const double *__restrict__ Xr = Xs + row0;
            double ca = 1.192611307487823e-07, cb = 2.409383341728244e-06;
            asm volatile("" : "+s"(ca), "+v"(cb));
            // same pipeline as the table form: the next point's row is requested while this one is worked
            // on, the stream one float4 ahead
            const int last = n_iter - 1;
            auto one_point = [&](const double (&rc)[D + 1], double (&rn)[D + 1], const double *__restrict__ next,
                                 float vf) {
#pragma unroll
                for (int d = 0; d <= D; ++d) rn[d] = next[d];
                __builtin_amdgcn_sched_barrier(0);
                double t = qs + rc[D];
#pragma unroll
                for (int d = 0; d < D; ++d) t = fma(xs[d], rc[d], t);
                const double k = exp2_poly(t, ca, cb);
                const double vk = (double)vf * k;
                u += vk;
                if (JAC) {
#pragma unroll
                    for (int d = 0; d < D; ++d) G[d] = fma(vk, rc[d], G[d]);
                }
                __builtin_amdgcn_sched_barrier(0);
            };
            double ra[D + 1], rb[D + 1];
#pragma unroll
            for (int d = 0; d <= D; ++d) ra[d] = Xr[d];
            auto four_points = [&](const v4f vv, int n4) {
                const double *__restrict__ r = Xr + (size_t)(n4 * 4) * (D + 1);
                one_point(ra, rb, r + 1 * (D + 1), vv.x);
                one_point(rb, ra, r + 2 * (D + 1), vv.y);
                one_point(ra, rb, r + 3 * (D + 1), vv.z);
                one_point(rb, ra, n4 < last ? r + 4 * (D + 1) : Xr, vv.w);
            };
            v4f va = stream_load(vdesc, voff, 0u);
            for (int n4 = 0; n4 < n_iter; n4 += 2) {
                const v4f vb = stream_load(vdesc, voff, (unsigned)(n4 + 1) * vstep);
                four_points(va, n4);
                va = stream_load(vdesc, voff, (unsigned)(n4 + 2 < last ? n4 + 2 : last) * vstep);
                four_points(vb, n4 + 1);
            }
        }
        combine_waves<D, JAC, RC>(red, wave, lane, live, out, B, false, u, G);
    } else {
        // ---------------- random-feature unit: CL features of output m -------------------
        const int gg = group - M * ngk;
        const int m = gg / ngl, c = 4 * (gg - m * ngl) + wave;
        const int n_iter = c < ncl ? CL / 4 : 0;
        const double *__restrict__ Or = Os + (BAGEL_SAME_ROWS ? 0 : ((size_t)m * Lp + (size_t)c * CL) * (D + 1));
        const unsigned wstep = (unsigned)S * (unsigned)sizeof(float4);
        const __amdgpu_buffer_rsrc_t wdesc =
            stream_descriptor(w4 + ((size_t)m * (Lp / 4) + (size_t)c * (CL / 4)) * S, (size_t)(CL / 4) * wstep);
        const unsigned woff = (unsigned)sidx * (unsigned)sizeof(float4);
        float p = 0.0f;
        if (JAC) {
            // The Jacobian sums of the feature part, G[b][d] = sum_l (w_l sin z_l) omega_ld, tolerate
            // float32 (no cancellation: w has random signs), so they run on the matrix cores as rank-1
            // updates: v_mfma_f32_4x4x1 (16 blocks) multiplies, within every group of four lanes, the A
            // values of the four lanes (here: w sin z of four trajectories) with the B values of the four
            // lanes (here: omega_ld for d = 4 q + lane % 4) and adds the 4 x 4 products to four registers
            // (register i of lane 4 g + j: trajectory 4 g + i, column 4 q + j).  One instruction takes the
            // issue time of two vector FMAs and replaces four of them (and the float64 conversion).
            // Of holds omega / (2 pi) in float32 in the order the B operand needs: per four features and
            // lane class j, NQ float4 (feature 0..3 of column 4 q + j), read through a buffer load whose
            // lane offset is constant; columns >= D are zero.
            const unsigned ostep = 64u * NQ;            // bytes per four features
            const __amdgpu_buffer_rsrc_t odesc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float4 *>(Of + ((size_t)m * (Lp / 4) + (size_t)c * (CL / 4)) * 4 * NQ), 0,
                (int)((size_t)(CL / 4) * ostep), 0x00020000);
            const unsigned ooff = (unsigned)(lane & 3) * (16u * NQ);
            f4v acc[NQ];
#pragma unroll
            for (int qd = 0; qd < NQ; ++qd) acc[qd] = f4v{0.0f, 0.0f, 0.0f, 0.0f};
            const int last = n_iter - 1;         // CL is a multiple of 8: two float4 per trip, no branch
            auto one_feature = [&](const double (&rc)[D + 1], double (&rn)[D + 1], const double *__restrict__ next,
                                   float wf, const v4f (&bq)[NQ], int j) {
#pragma unroll
                for (int d = 0; d <= D; ++d) rn[d] = next[d];
                __builtin_amdgcn_sched_barrier(0);
                // product first, phase offset last: both are scalar operands, and an FMA takes only one
                double z = x[0] * rc[0];
#pragma unroll
                for (int d = 1; d < D; ++d) z = fma(x[d], rc[d], z);
                z += rc[D];
                // z is the phase in revolutions; its fractional part is exact in float64 and the
                // hardware sin / cos take revolutions (absolute error about one float32 ulp)
                const float y = (float)__builtin_amdgcn_fract(z);
                const float sn = __builtin_amdgcn_sinf(y);
                const float cs = __builtin_amdgcn_cosf(y);
                p = fmaf(wf, cs, p);
                const float ws = wf * sn;
#pragma unroll
                for (int qd = 0; qd < NQ; ++qd)
                    acc[qd] = __builtin_amdgcn_mfma_f32_4x4x1f32(ws, bq[qd][j], acc[qd], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            };
            double fa[D + 1], fb[D + 1];
#pragma unroll
            for (int d = 0; d <= D; ++d) fa[d] = Or[d];
            // four features whose weights are in ww; `next` receives the stream's float4 of step l4_next,
            // requested after this step's B operands (loads return in order: the wait for the operands,
            // which hit in cache, must not include the stream's trip to HBM)
            auto four_features = [&](const v4f ww, int l4, v4f &next, int l4_next) {
                v4f bq[NQ];
#pragma unroll
                for (int qd = 0; qd < NQ; ++qd)
                    bq[qd] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(odesc, ooff + 16u * qd, (unsigned)l4 * ostep, 0));
                __builtin_amdgcn_sched_barrier(0);
                next = stream_load(wdesc, woff, (unsigned)l4_next * wstep);
                __builtin_amdgcn_sched_barrier(0);
                // each feature's row was requested while the previous feature was being worked on (see the
                // kernel-row loop); the request after the unit's last row stays inside the table
                const double *__restrict__ r = Or + (size_t)(l4 * 4) * (D + 1);
                one_feature(fa, fb, r + 1 * (D + 1), ww.x, bq, 0);
                one_feature(fb, fa, r + 2 * (D + 1), ww.y, bq, 1);
                one_feature(fa, fb, r + 3 * (D + 1), ww.z, bq, 2);
                one_feature(fb, fa, l4 < last ? r + 4 * (D + 1) : Or, ww.w, bq, 3);
            };
            // the stream of w one float4 ahead in alternating register sets, as in the kernel-row loop
            v4f wa = stream_load(wdesc, woff, 0u), wb = wa;
            for (int l4 = 0; l4 < n_iter; l4 += 2) {
                four_features(wa, l4, wb, l4 + 1);
                four_features(wb, l4 + 1, wa, l4 + 2 < last ? l4 + 2 : last);
            }
            // every wave, wave 0 included, hands its sums over through LDS: that is also the transposition
            // from the accumulator layout (lane = column, register = trajectory) to lane = trajectory
            const int slot = (wave + 3) & 3;
            red[slot][0][lane] = (double)p;
#pragma unroll
            for (int qd = 0; qd < NQ; ++qd) {
                const int d = 4 * qd + (lane & 3);
                if (d < D) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) red[slot][1 + d][(lane & ~3) + i] = (double)acc[qd][i];
                }
            }
            double u = 0.0, G[D];
            combine_waves<D, JAC, RC>(red, wave, lane, live, out, B, true, u, G);
        } else {
            // value only: the same pipeline without the Jacobian sums
            const int last = n_iter - 1;
            auto one_feature = [&](const double (&rc)[D + 1], double (&rn)[D + 1], const double *__restrict__ next,
                                   float wf) {
#pragma unroll
                for (int d = 0; d <= D; ++d) rn[d] = next[d];
                __builtin_amdgcn_sched_barrier(0);
                double z = x[0] * rc[0];
#pragma unroll
                for (int d = 1; d < D; ++d) z = fma(x[d], rc[d], z);
                z += rc[D];
                const float y = (float)__builtin_amdgcn_fract(z);
                p = fmaf(wf, __builtin_amdgcn_cosf(y), p);
                __builtin_amdgcn_sched_barrier(0);
            };
            double fa[D + 1], fb[D + 1];
#pragma unroll
            for (int d = 0; d <= D; ++d) fa[d] = Or[d];
            auto four_features = [&](const v4f ww, int l4) {
                const double *__restrict__ r = Or + (size_t)(l4 * 4) * (D + 1);
                one_feature(fa, fb, r + 1 * (D + 1), ww.x);
                one_feature(fb, fa, r + 2 * (D + 1), ww.y);
                one_feature(fa, fb, r + 3 * (D + 1), ww.z);
                one_feature(fb, fa, l4 < last ? r + 4 * (D + 1) : Or, ww.w);
            };
            v4f wa = stream_load(wdesc, woff, 0u);
            for (int l4 = 0; l4 < n_iter; l4 += 2) {
                const v4f wb = stream_load(wdesc, woff, (unsigned)(l4 + 1) * wstep);
                four_features(wa, l4);
                wa = stream_load(wdesc, woff, (unsigned)(l4 + 2 < last ? l4 + 2 : last) * wstep);
                four_features(wb, l4 + 1);
            }
            double u = (double)p, G[D];
            combine_waves<D, JAC, RC>(red, wave, lane, live, out, B, false, u, G);
        }
    }
}

template <int D, bool JAC, bool NEAR>
void launch_variant(bagel_ctx *c, float *prev_jac)
{
    dim3 grid((c->dm.B + 63) / 64, c->groups + (prev_jac ? c->M : 0));
    const int per_sample = c->dm.B / c->dm.S;
    const jac_sums prev = {c->part_alt, c->xbuf_alt, c->A, c->amp, prev_jac};
    hipLaunchKernelGGL((gp_step_kernel<D, JAC, NEAR>), grid, dim3(BAGEL_BLOCK), 0, c->stream, c->Xs, c->Xn, c->Os,
                       reinterpret_cast<const float4 *>(c->Of), c->A, c->v4, c->w4, c->xbuf, c->part, c->exp_tab,
                       c->near_ok, c->dm.B, c->dm.S, per_sample, c->Np, c->Lp, c->CK, c->CL, c->nck, c->ncl, c->M, prev);
}

template <int D>
hipError_t launch_d(bagel_ctx *c, bool jac, float *prev_jac)
{
    if (c->exp_table) {
        if (jac) launch_variant<D, true, true>(c, prev_jac);
        else launch_variant<D, false, true>(c, prev_jac);
    } else {
        if (jac) launch_variant<D, true, false>(c, prev_jac);
        else launch_variant<D, false, false>(c, prev_jac);
    }
    return hipGetLastError();
}

}  // namespace

int bagel_env_int(const char *name, int dflt)
{
    const char *s = getenv(name);
    if (!s || !*s) return dflt;
    const int v = atoi(s);
    return v > 0 ? v : dflt;
}

// Work decomposition of one sample evaluation (sets CK, CL, nck, ncl, Np, Lp, units, groups and the
// exp2 form from dm, D, M); returns a message if the problem cannot be decomposed.
const char *bagel_plan_sample_eval(bagel_ctx *c)
{
    // work decomposition of one sample evaluation: power-of-two chunk of training points / features
    const bagel_dims *dims = &c->dm;
    const int B = dims->B, N = dims->N, L = dims->L, M = c->M;
    const int64_t tb = (B + BAGEL_BLOCK - 1) / BAGEL_BLOCK;
    const int64_t items = (int64_t)(N + L) * M * tb;
    const int target = bagel_env_int("BAGEL_TARGET_WGS", 4096);
    int chunk = 1024;
    while (chunk > 32 && items / chunk < target) chunk /= 2;
    // Longer units for the training points when there are plenty of them (fewer partial sums), shorter
    // ones for the features of a large problem: workgroups are dispatched in grid order, training-point
    // units first, so short feature units at the end fill the tail of the launch.  Measured on MI355X:
    // stress 0.650 ms per launch at (CK, CL) = (1024, 512), 0.628 ms at (1024, 256); the large-policy
    // step 140.6 ms at (128, 64), 136.8 ms at (256, 64).
    // A launch that stays under the target even with the smallest chunk has only a handful of waves per
    // SIMD, and the longest of them sets its duration (measured: launch time grows in proportion to
    // CK), so its units are kept short and alike: medium 10.7 ms per call at (128, 32), 9.7 ms at
    // (64, 64); small 3.78 ms at (64, 32), 3.46 ms at (32, 32).  (Staging the operand rows through LDS
    // and look-ahead loads of the stream changed nothing there: those launches are not latency-bound.)
    const bool small_launch = chunk == 32 && items / chunk < target;
    const int ck_default = small_launch ? (N / chunk >= 64 ? 64 : 32)
                                        : (N / chunk >= 32 ? 4 * chunk : (N / chunk >= 16 ? 2 * chunk : chunk));
    const int cl_default = small_launch ? (N / chunk >= 64 ? 64 : 32)
                                        : ((chunk >= 512 && L / chunk >= 8) ? chunk / 2 : chunk);
    c->CK = bagel_env_int("BAGEL_CK", ck_default);
    c->CL = bagel_env_int("BAGEL_CL", cl_default);
    c->CK = (c->CK + 7) & ~7;         // the sample-evaluation loops take two float4 (eight points) per trip
    c->CL = (c->CL + 7) & ~7;
    c->nck = (N + c->CK - 1) / c->CK;
    c->ncl = (L + c->CL - 1) / c->CL;
    c->Np = c->nck * c->CK;
    c->Lp = c->ncl * c->CL;
    c->units = M * (c->nck + c->ncl);
    c->groups = M * ((c->nck + 3) / 4 + (c->ncl + 3) / 4);
    // The table form of the kernel-row loop (gp_step.hip) pays once the launch has a few workgroups per
    // compute unit; below that its extra set-up per workgroup (the table copy) and the wait counter its
    // LDS read shares with the scalar loads cost more than its five fewer instructions per training point
    // save.  Measured on MI355X, table vs general form, per launch: stress (4608 workgroups) 0.561 vs
    // 0.60 ms; large policy (3072) 83.7 vs 86.4 us; medium (1280) 20.9 vs 22.4 us; small (192) 9.6 vs 9.2 us.
    {
        const int64_t wgs = (int64_t)((B + 63) / 64) * c->groups;
        const int tab = bagel_env_int("BAGEL_EXP_TABLE", 0);         // 1: off, 2: on, otherwise by launch size
        c->exp_table = tab == 2 ? true : (tab == 1 ? false : wgs >= 1024);
    }
    if (c->units > 65535 - BAGEL_MAX_STATE) return "too many work units (M * (N + L) / 32 must stay below 65527)";
    return nullptr;
}

hipError_t bagel_launch_gp_step(bagel_ctx *c, bool jac, float *prev_jac)
{
    switch (c->D) {
#define CASE(n) case n: return launch_d<n>(c, jac, prev_jac);
        CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12)
        CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
    }
    return hipErrorInvalidValue;
}

hipError_t bagel_launch_jac_reduce(bagel_ctx *c, float *jdst)
{
    const jac_sums j = {c->part, c->xbuf, c->A, c->amp, jdst};
    hipLaunchKernelGGL(jac_reduce_kernel, dim3((c->dm.B + 63) / 64, c->M), dim3(BAGEL_BLOCK), 0, c->stream, j, c->dm.B, c->D,
                       c->M, (c->nck + 3) / 4, (c->ncl + 3) / 4);
    return hipGetLastError();
}
