// Lane-per-trajectory kernels at the edges of a rollout: initial state,
// the final loss reduction (Algorithm 1: loss = mean over trajectories of the summed cost), and the
// plumbing of bagel_sample_eval (reduction of the partial sums of one sample evaluation on its own;
// inside a rollout that reduction is part of the end-of-step kernel).
// All per-trajectory arrays are laid out [component][B] so that a wave reads consecutive
// trajectories.
#include "bagel_internal.h"

namespace {

constexpr double LN2 = 0.69314718055994530942;
constexpr double TWO_PI = 6.28318530717958647693;

struct lane_args {
    int B, D, M, ds, da, dg, H;
    int nck, ncl;                // groups of work units per output: training points, features
    int cost_kind;
    float sigma_r, act_bound;
    int tracked[8];
    float q[8];
    const double *A, *amp, *part;
    double *xbuf, *lpt;
    float *tape_s;
};

// Add up the partial sums of one sample evaluation in unit order and finish value and Jacobian.
// One thread per (trajectory, output m, component): component 0 is the value
//   f[m] = amp_m * sum_c p_c + sum_c u_c,
// component 1+d the Jacobian entry
//   J[m][d] = -amp_m (2 pi) sum_c Gr_c[d] + ln2 (sum_c Gk_c[d] - log2(e)/l_md^2 x_d sum_c u_c).
// f goes to fbuf[m][b] (float64); J[m][d] to jdst[(m*D+d)*js_i + b*js_b] (float32), which is either a
// tape slot ([M][D][B]) or a caller array ([B][M][D]).
__global__ __launch_bounds__(BAGEL_BLOCK) void finalize_kernel(lane_args a, int ncomp, double *__restrict__ fbuf,
                                                               float *__restrict__ jdst, long js_i, long js_b)
{
    const int b = blockIdx.x * BAGEL_BLOCK + threadIdx.x;
    if (b >= a.B) return;
    const int m = blockIdx.y / ncomp, comp = blockIdx.y - m * ncomp;
    const size_t stride = (size_t)(1 + a.D) * a.B;
    const double *pk = a.part + (size_t)(m * a.nck) * stride + b;
    const double *pr = a.part + (size_t)(a.M * a.nck + m * a.ncl) * stride + b;
    double u = 0.0;
    for (int c = 0; c < a.nck; ++c) u += pk[c * stride];
    const double amp = a.amp[m];
    if (comp == 0) {
        double p = 0.0;
        for (int c = 0; c < a.ncl; ++c) p += pr[c * stride];
        fbuf[(size_t)m * a.B + b] = amp * p + u;
    } else {
        const int d = comp - 1;
        double gk = 0.0, gr = 0.0;
        for (int c = 0; c < a.nck; ++c) gk += pk[c * stride + (size_t)comp * a.B];
        for (int c = 0; c < a.ncl; ++c) gr += pr[c * stride + (size_t)comp * a.B];
        const double x = a.xbuf[(size_t)d * a.B + b];
        const double J = -amp * TWO_PI * gr + LN2 * (gk - a.A[m * a.D + d] * x * u);
        jdst[(long)(m * a.D + d) * js_i + (long)b * js_b] = (float)J;
    }
}

__global__ __launch_bounds__(BAGEL_BLOCK) void init_state_kernel(lane_args a, const float *__restrict__ s0,
                                                                 const float *__restrict__ goals0,
                                                                 float *__restrict__ states_out,
                                                                 float *__restrict__ h0_slot)
{
    const int b = blockIdx.x * BAGEL_BLOCK + threadIdx.x;
    if (b >= a.B) return;
    for (int i = 0; i < a.ds; ++i) {
        const float v = s0[(size_t)b * a.ds + i];
        a.xbuf[(size_t)i * a.B + b] = (double)v;
        if (a.tape_s) a.tape_s[(size_t)i * a.B + b] = v;
        if (states_out) states_out[(size_t)b * a.ds + i] = v;
        h0_slot[(size_t)i * a.B + b] = v;
    }
    for (int j = 0; j < a.dg; ++j) h0_slot[(size_t)(a.ds + j) * a.B + b] = goals0[(size_t)b * a.dg + j];
    a.lpt[b] = 0.0;
}

// loss = (1/B) sum_b lpt[b], summed in a fixed tree order by one workgroup
__global__ __launch_bounds__(1024) void finish_loss_kernel(const double *__restrict__ lpt, int B,
                                                           float *__restrict__ loss,
                                                           float *__restrict__ loss_per_traj)
{
    __shared__ double sh[1024];
    double acc = 0.0;
    for (int b = threadIdx.x; b < B; b += 1024) {
        const double v = lpt[b];
        acc += v;
        if (loss_per_traj) loss_per_traj[b] = (float)v;
    }
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[0] = (float)(sh[0] / (double)B);
}

// bagel_sample_eval plumbing: phase 0 loads x[B][D] into xbuf; phase 1 writes f[B][M] from fbuf.
__global__ __launch_bounds__(BAGEL_BLOCK) void eval_io_kernel(lane_args a, int phase, const float *__restrict__ xin,
                                                              const double *__restrict__ fbuf,
                                                              float *__restrict__ f_out)
{
    const int b = blockIdx.x * BAGEL_BLOCK + threadIdx.x;
    if (b >= a.B) return;
    if (phase == 0) {
        for (int d = 0; d < a.D; ++d) a.xbuf[(size_t)d * a.B + b] = (double)xin[(size_t)b * a.D + d];
        return;
    }
    for (int m = 0; m < a.M; ++m) f_out[(size_t)b * a.M + m] = (float)fbuf[(size_t)m * a.B + b];
}

lane_args make_args(const bagel_ctx *c)
{
    lane_args a;
    a.B = c->dm.B; a.D = c->D; a.M = c->M; a.ds = c->dm.d_s; a.da = c->dm.d_a; a.dg = c->dm.d_g; a.H = c->dm.H;
    a.nck = (c->nck + 3) / 4; a.ncl = (c->ncl + 3) / 4;
    a.cost_kind = c->dm.cost_kind; a.sigma_r = c->dm.sigma_r; a.act_bound = c->dm.act_bound;
    for (int j = 0; j < 8; ++j) { a.tracked[j] = c->dm.tracked[j]; a.q[j] = c->dm.q[j]; }
    a.A = c->A; a.amp = c->amp; a.part = c->part;
    a.xbuf = c->xbuf; a.lpt = c->lpt;
    a.tape_s = nullptr;
    return a;
}

inline dim3 lane_grid(const bagel_ctx *c) { return dim3((c->dm.B + BAGEL_BLOCK - 1) / BAGEL_BLOCK); }

}  // namespace

static inline float *slot_ptr(float *base, int slot, int width, int B) { return base + (size_t)slot * width * B; }

hipError_t bagel_launch_init_state(bagel_ctx *c, const float *s0, const float *goals, float *states_out,
                                   bool tape)
{
    lane_args a = make_args(c);
    a.tape_s = tape ? c->tape_s : nullptr;
    hipLaunchKernelGGL(init_state_kernel, lane_grid(c), dim3(BAGEL_BLOCK), 0, c->stream, a, s0, goals, states_out,
                       slot_ptr(c->tape_h[0], 0, c->d_in, c->dm.B));
    return hipGetLastError();
}

hipError_t bagel_launch_finish_loss(bagel_ctx *c, float *loss, float *loss_per_traj)
{
    hipLaunchKernelGGL(finish_loss_kernel, dim3(1), dim3(1024), 0, c->stream, c->lpt, c->dm.B, loss, loss_per_traj);
    return hipGetLastError();
}

hipError_t bagel_launch_eval_io(bagel_ctx *c, int phase, const float *x, float *f)
{
    lane_args a = make_args(c);
    hipLaunchKernelGGL(eval_io_kernel, lane_grid(c), dim3(BAGEL_BLOCK), 0, c->stream, a, phase, x, c->fbuf, f);
    return hipGetLastError();
}

// slot >= 0: Jacobian into that tape slot; slot < 0: into jac_out[B][M][D] (may be null: value only)
hipError_t bagel_launch_finalize(bagel_ctx *c, bool jac, int slot, float *jac_out)
{
    lane_args a = make_args(c);
    const int ncomp = jac ? 1 + c->D : 1;
    dim3 grid((c->dm.B + BAGEL_BLOCK - 1) / BAGEL_BLOCK, c->M * ncomp);
    float *jdst = nullptr;
    long js_i = 0, js_b = 0;
    if (jac) {
        if (slot >= 0) { jdst = slot_ptr(c->tape_J, slot, c->M * c->D, c->dm.B); js_i = c->dm.B; js_b = 1; }
        else { jdst = jac_out; js_i = 1; js_b = (long)c->M * c->D; }
    }
    hipLaunchKernelGGL(finalize_kernel, grid, dim3(BAGEL_BLOCK), 0, c->stream, a, ncomp, c->fbuf, jdst, js_i, js_b);
    return hipGetLastError();
}
