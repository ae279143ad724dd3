// Internal declarations shared by the translation units of libbagel.so.
// Nothing here is part of the public ABI (see include/bagel.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bagel.h"

#define BAGEL_BLOCK 256          // threads per workgroup in the lane-per-trajectory kernels
#define BAGEL_MAX_D 16

struct bagel_ctx {
    bagel_dims dm;
    int D, M, P, d_in;
    int n_layers;                // n_hidden + 1
    int width[4];                // d_in, hidden..., d_a
    int w_off[3], b_off[3];      // offsets of W_l and b_l inside theta
    hipStream_t stream;
    bool prepared;
    char err[512];
    int64_t bytes;

    // ---- model, internal layout --------------------------------------------------------
    int Np, Lp;                  // N and L rounded up to a whole number of chunks
    int CK, CL;                  // training points / features per work unit (multiples of 8)
    int nck, ncl;                // chunks per output
    int units;                   // M * (nck + ncl)
    int groups;                  // M * (ceil(nck/4) + ceil(ncl/4)): four units per workgroup and partial sum
    bool exp_table;              // sample-evaluation kernel with the table form of the kernel-row loop (large launches)
    double *Xs;                  // [M][Np][D+1]: log2(e)/l_md^2 * X_nd, then log2(alpha_m^2) - 1/2 sum_d log2(e)/l_md^2 X_nd^2
    double *Os;                  // [M][Lp][D+1]: omega_mld / (2 pi) (revolutions per unit x_d), then phase / (2 pi)
    float *Of;                   // [M][Lp/4][4][NQ][4], NQ = ceil(D/4): omega / (2 pi) in float32 in the order of the matrix-core
                                 // B operand of the feature Jacobian: entry (m, l4, j, q, f) is column 4q+j of feature 4 l4 + f
    double *A;                   // [M][D]: log2(e) / l_md^2
    double *amp;                 // [M]: sqrt(2 alpha_m^2 / L)
    double *Xn;                  // [M][Np][D+1]: as Xs, last entry + 6144 (the table form's rows; see gp_step.hip)
    int *near_ok;                // [1]: 1 if every training point and alpha^2 are inside the table form's range
    double *exp_tab;             // [256]: -2^(i/256) with i << 12 subtracted from its high word (see gp_step.hip)
    float4 *v4;                  // [M][Np/4][S]: four consecutive training points of one sample
    float4 *w4;                  // [M][Lp/4][S]

    // ---- per-step workspace (lane = trajectory, arrays are [component][B]) ---------------
    double *xbuf;                // [D][B]   GP input of the current step; rows 0..d_s-1 are the state (float64)
    double *part;                // [groups][1+D][B] partial sums of the current step
    double *xbuf_alt, *part_alt; // the same two buffers for the neighbouring step: a rollout swaps them with
                                 // xbuf / part after every step, so that the Jacobian sums of step t-1 can be
                                 // added up while step t is evaluated (both need their own inputs and sums)
    double *lpt;                 // [B] running cost per trajectory
    double *lam;                 // [d_s][B] adjoint of the state between the segments of a checkpointed sweep
    double *fbuf;                // [M][B] sample values of the current step, summed over work units

    // ---- tape: activations and adjoints have T_tape slots (H, or ckpt_interval when checkpointing:
    // they are rebuilt segment by segment); states and Jacobians are kept for the whole horizon
    int T_tape;
    float *tape_s;               // [H+1][d_s][B]
    float *tape_J;               // [H][M][D][B]
    float *tape_h[3];            // activations feeding layer l: [T][width[l]][B]
    float *tape_a;               // [T][d_a][B] policy output (after tanh, before scaling, if bounded)
    float *tape_d[3];            // adjoint of the pre-activation of layer l: [T][width[l+1]][B]
    // With checkpointing the three per-segment tapes above exist twice and tape_h / tape_a / tape_d point
    // to the set in use (set 0 outside the backward pass): while the sweep walks one segment on the
    // context's stream, the policy replay of the segment before it and the weight gradient of the
    // segment after it run on `side`, each on the other set.  Without checkpointing set 1 is empty.
    float *tape_h_set[2][3], *tape_a_set[2], *tape_d_set[2][3];
    hipStream_t side;            // null without checkpointing
    hipEvent_t ev_fork, ev_join, ev_replay[2], ev_sweep[2];

    // ---- parameters and gradient -----------------------------------------------------------
    float *wpad_f, *wpad_b;      // zero-padded weights: forward [out pad 32][in pad 32], backward [in pad 32][out pad 32]
    int wpf_off[3], wpf_rp[3], wpf_kp[3];
    int wpb_off[3], wpb_rp[3], wpb_kp[3];
    float *gsplit;               // [ksplit][P] split-contraction partial weight gradients
    double *gacc;                // [P] gradient accumulated over segments
    float *gtheta;               // [P] gradient of the current iteration of bagel_optimize
    int ksplit;
    int wg_lds_raised;           // bit i: the dynamic-LDS limit of weight-gradient kernel instance i has been raised on this context's device

    // ---- per-step posterior sampler (buffers allocated by the first bagel_prepare_posterior) -----
    bool post_prepared;
    int post_Np;                 // N rounded up to a multiple of 64
    double post_sf2[8];          // alpha_m^2
    double *post_alpha;          // [M][post_Np]           K_hat^-1 y, zero on the padding
    double *post_Kinv;           // [M][post_Np][post_Np]  K_hat^-1
    double *post_Kx;             // [M][post_Np][B]: kernel rows at the current inputs
    double *post_sums;           // [M][post_Np/64][2(1+D)][B]: per-tile sums of the moments
    const float *cur_xi;         // draws of the rollout in progress (null: pathwise sampler)

    // ---- set-up calls (prepare.hip): side streams and float64 work space, made by the first of them --
    void *setup;

    // ---- measurement hooks -------------------------------------------------------------------
    int prof_every, prof_seen, prof_used;
    hipEvent_t *prof_ev;         // 2 * BAGEL_PROF_MAX events, created on enable
};
#define BAGEL_PROF_MAX 4096

#define BAGEL_FAIL(ctx, code, ...)                                   \
    do {                                                             \
        snprintf((ctx)->err, sizeof((ctx)->err), __VA_ARGS__);      \
        return (code);                                               \
    } while (0)

#define BAGEL_HIP(ctx, call)                                                                   \
    do {                                                                                       \
        hipError_t e__ = (call);                                                               \
        if (e__ != hipSuccess)                                                                 \
            BAGEL_FAIL(ctx, BAGEL_EHIP, "%s failed: %s", #call, hipGetErrorString(e__));      \
    } while (0)

// ---- gp_step.hip -------------------------------------------------------------------------
// Integer from the environment (the overrides documented in bagel.h), or dflt if unset or not positive.
int bagel_env_int(const char *name, int dflt);
// Work decomposition of one sample evaluation (sets CK, CL, nck, ncl, Np, Lp, units, groups and the
// exp2 form from dm, D, M); returns a message, a string literal, if the problem cannot be decomposed.
const char *bagel_plan_sample_eval(bagel_ctx *ctx);
// One evaluation of all function samples at xbuf: partial sums per work unit into ctx->part.
// prev_jac: if not null, the same launch also adds up the Jacobian sums of the previous step (in
// ctx->part_alt, evaluated at ctx->xbuf_alt) into prev_jac[M][D][B] (a slot of the Jacobian tape).
hipError_t bagel_launch_gp_step(bagel_ctx *ctx, bool jac, float *prev_jac);
// The Jacobian sums in ctx->part (evaluated at ctx->xbuf) added up into jdst[M][D][B], on their own.
hipError_t bagel_launch_jac_reduce(bagel_ctx *ctx, float *jdst);

// ---- model.hip ---------------------------------------------------------------------------
hipError_t bagel_launch_build_model(bagel_ctx *ctx, const float *X, const float *ell, const float *sf2,
                                    const float *omega, const float *phase);
hipError_t bagel_launch_pack_samples(bagel_ctx *ctx, const float *w, const float *v);

// ---- lane.hip ----------------------------------------------------------------------------
hipError_t bagel_launch_init_state(bagel_ctx *ctx, const float *s0, const float *goals, float *states_out,
                                   bool tape);
hipError_t bagel_launch_finish_loss(bagel_ctx *ctx, float *loss, float *loss_per_traj);
hipError_t bagel_launch_eval_io(bagel_ctx *ctx, int phase, const float *x, float *f);
// add up the per-unit partial sums: value into fbuf, Jacobian into tape slot `slot` (or jac_out if slot < 0)
hipError_t bagel_launch_finalize(bagel_ctx *ctx, bool jac, int slot, float *jac_out);

// ---- policy.hip --------------------------------------------------------------------------
hipError_t bagel_launch_pack_theta(bagel_ctx *ctx, const float *theta);
hipError_t bagel_launch_policy_forward(bagel_ctx *ctx, int slot, const float *theta);
// after the sample evaluation of step t: add up the value sums in ctx->part, advance the state (read from
// ctx->xbuf, written to ctx->xbuf_alt), cost against goals[t], state tape, and the policy of step t+1
// into tape slot next_slot, its action into ctx->xbuf_alt (no policy if t is the last step or
// next_slot < 0).  The caller swaps xbuf / xbuf_alt and part / part_alt afterwards.  The Jacobian sums
// are not touched (bagel_launch_gp_step / bagel_launch_jac_reduce), except with direct: ctx->part
// then holds final values [m][1+D][B], whose Jacobian goes to tape slot `slot` here if jac.
hipError_t bagel_launch_step_tail(bagel_ctx *ctx, int t, int slot, int next_slot, bool jac, bool add_cost,
                                  bool write_tape_s, const float *theta, const float *goals,
                                  float *states_out, bool direct);
// activation tape of steps t0 .. t1-1 (slots 0 .. t1-t0-1) rebuilt from the kept states
hipError_t bagel_launch_policy_replay(bagel_ctx *ctx, int t0, int t1, const float *theta, const float *goals);
// backward sweep over steps t_hi-1 .. t_lo (tape slot of step k is k - t_lo); grad_s0 is written when t_lo == 0
hipError_t bagel_launch_backward_sweep(bagel_ctx *ctx, int t_lo, int t_hi, const float *goals, float *grad_s0);
hipError_t bagel_launch_weight_grad(bagel_ctx *ctx, int n_slots, bool accumulate, float *grad_theta);
hipError_t bagel_launch_adam(bagel_ctx *ctx, float *theta, const float *grad, float *m, float *v, int count, double lr,
                             double beta1, double beta2, double eps, double corr1, double corr2);

// ---- posterior.hip ------------------------------------------------------------------------
// mu + sqrt(var) xi and its Jacobian for every trajectory and output at xbuf, into ctx->part as
// [m][1+D][B] (final values, not partial sums)
hipError_t bagel_launch_posterior_step(bagel_ctx *ctx, bool jac, const float *xi_t);

// ---- prepare.hip -------------------------------------------------------------------------
// v = (K + noise I)^-1 (y - Phi w - eps) for every sample, float64 inside; packs v into ctx->v4
// and optionally writes float32 v_out[S][M][N].  Returns a BAGEL_* code and sets ctx->err.
int bagel_prepare_impl(bagel_ctx *ctx, const float *X, const float *y, const float *ell, const float *sf2,
                       const float *sn2, const float *omega, const float *phase, const float *w,
                       const float *eps, float *v_out);

// K_hat^-1 and K_hat^-1 y of every output into ctx->post_Kinv / post_alpha (float64)
int bagel_prepare_posterior_impl(bagel_ctx *ctx, const float *X, const float *y, const float *ell, const float *sf2,
                                 const float *sn2);
// release the side streams and work space of the set-up calls (bagel_destroy)
void bagel_release_setup(bagel_ctx *ctx);
// C (+)= alpha * A * B in float64 with element strides (see dgemm_kernel); overwrite: C = alpha * A * B
void bagel_dgemm(hipStream_t st, int Mr, int Nc, int Kd, double alpha, const double *A, long sai, long sak,
                 const double *Bm, long sbk, long sbj, double *Cm, long ldc, bool overwrite);
// lml[iters][M] and grad[M][D+2] of the log hyper-parameters log_hyp[M][D+2]; n_iters > 0: Adam fit in place
int bagel_hyper_impl(bagel_ctx *ctx, const float *X, const float *y, float *log_hyp, float *lml, float *grad,
                     float *adam_m, float *adam_v, int n_iters, int first_step, double lr, double beta1, double beta2,
                     double eps);
