/*
 * bagel.h - C ABI of libbagel.so: batched Monte-Carlo rollouts of a tanh-MLP
 * policy through pathwise-sampled Gaussian-process dynamics on one MI355X
 * (gfx950), and the reverse-mode gradient of the mean trajectory cost with
 * respect to the policy parameters (arXiv 2202.13638, Algorithm 1: forward
 * pass, loss, backward pass).
 *
 * Model (per GP output m = 0..d_s-1, one independent GP per state increment,
 * Sec. III-A):
 *   kernel      k_m(x,x') = signal_var[m] * exp(-1/2 sum_d (x_d-x'_d)^2 / lengthscale[m][d]^2)   eq. (4)
 *   features    phi_m(x)_l = sqrt(2 signal_var[m] / L) * cos(omega[m][l] . x + phase[m][l])
 *   sample s    f_sm(x) = phi_m(x)^T w[s][m] + k_m(x, X)^T v[s][m],
 *               v[s][m] = (K_m + noise_var[m] I)^-1 (y[m] - Phi_m w[s][m] - eps[s][m])            K_hat below eq. (3)
 * Rollout (Algorithm 1; trajectory b uses sample b / (B / S)):
 *   a_t = pi_theta([s_t ; g_t]),  x_t = [s_t ; a_t],  s_{t+1} = s_t + f_s(x_t),
 *   c_{t+1} = sum_j q[j] (s_{t+1}[tracked[j]] - g_t[j])^2            (cost_kind 0)
 *           = -exp(-(1/(2 sigma_r^2)) * that sum)                      (cost_kind 1, eq. (8) as a cost)
 *   loss = (1/B) sum_b sum_{t=1..H} c_t                                eq. (10), (11)
 *
 * Conventions
 *   - Every array argument is a DEVICE pointer to memory owned by the caller, row-major
 *     with the extents given in brackets, float32 unless stated.  The library reads inputs
 *     and writes outputs on the stream passed to bagel_create; it never frees or keeps
 *     caller memory after a call returns, except that prepare/set_samples copy the model
 *     into context-owned buffers in an internal layout.
 *   - The rollout calls enqueue work and return; they do not synchronise the stream and
 *     allocate nothing.  Outputs are valid once the stream has drained.  What they enqueue is
 *     kernel launches only (no memset or copy nodes), so a call may be captured into a HIP graph on
 *     the context's stream and replayed; the graph then holds the argument pointers of that call.
 *   - The kernel-row contraction over the N training points is evaluated in float64
 *     (operands are the float32 inputs promoted exactly); everything at the interface is
 *     float32.
 *   - theta layout: for each layer in order, W[out][in] row-major then b[out].
 *     Layers: (d_s+d_g) -> hidden[0] (-> hidden[1]) -> d_a, tanh on hidden layers;
 *     output a = z if act_bound <= 0, else act_bound * tanh(z) (Sec. IV-A: bounded action).
 *   - No random numbers are drawn inside the library: omega, phase, w, eps are inputs.
 *   - Return value: 0 on success, a negative BAGEL_E* code otherwise; bagel_last_error
 *     gives a message.  NaN/Inf inputs are not screened; they propagate.
 *   - Range of the kernel row (eq. (4)): training inputs and GP inputs are expected within about
 *     400 length scales of the origin (sum_d x_d^2 / l_d^2 < 1.8e5; the paper's data are
 *     normalised).  A training point further out is dropped from the kernel row, and a trajectory
 *     further out sees a kernel row of zero; both are exact as long as the other side stays inside.
 *     (Within about 19 length scales - sum_d x_d^2 / l_d^2 < 346 for data and trajectory, signal
 *     variance within 2^-20 .. 2^20 - large launches take a faster form of the same arithmetic; outside
 *     they fall back by themselves, per group of 64 trajectories.  Results agree to rounding.)
 *   - The two samplers share the model tables of a context: bagel_prepare_samples / bagel_set_samples
 *     install the pathwise sampler and invalidate the posterior cache, bagel_prepare_posterior does
 *     the reverse.  Use two contexts to hold both.
 *   - One context must not be used from two threads at once.
 *
 * Tuning knobs (environment variables read once by bagel_create; the defaults are the measured best and
 * none of them changes results beyond the order of floating-point sums):
 *   BAGEL_CK, BAGEL_CL     training points / features per work unit of the sample evaluation (rounded
 *                          up to multiples of 8)
 *   BAGEL_TARGET_WGS       number of workgroups the default unit sizes aim for (default 4096)
 *   BAGEL_EXP_TABLE        1: always the general form of the kernel-row loop, 2: always the table form,
 *                          unset: by launch size
 *   BAGEL_KSPLIT           split of the weight-gradient contraction (default 256)
 */
#ifndef BAGEL_H
#define BAGEL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BAGEL_OK 0
#define BAGEL_EINVAL (-1)        /* null pointer, non-positive or unsupported dimension, S does not divide B ... */
#define BAGEL_ENOTPREPARED (-2)  /* rollout called before prepare_samples / set_samples */
#define BAGEL_ENOMEM (-3)        /* device allocation failed in bagel_create */
#define BAGEL_ENOTPD (-4)        /* K + noise_var I is not positive definite in float64 */
#define BAGEL_EHIP (-5)          /* a HIP runtime call failed */

#define BAGEL_MAX_STATE 8        /* d_s <= 8, d_a <= 8, d_g <= 8 */
#define BAGEL_MAX_HIDDEN 256     /* width of a hidden layer */

typedef struct bagel_ctx bagel_ctx; /* opaque; owns the model copy and all workspace */

typedef struct {
    int32_t d_s, d_a, d_g;   /* states, actions, tracked states (= goal dimension); D = d_s + d_a */
    int32_t N, L, S, B, H;   /* training points, features, function samples, trajectories, horizon;
                                1 <= S <= B and B % S == 0 */
    int32_t n_hidden;        /* 1 or 2 */
    int32_t hidden[2];
    float act_bound;         /* <= 0: linear output */
    int32_t tracked[8];      /* state index of goal component j, j < d_g */
    float q[8];              /* cost weight of goal component j */
    int32_t ckpt_interval;   /* 0: keep the whole tape in the gradient call; K > 0: gradient checkpointing
                                (Sec. IV-C: trading compute for memory): the activations and adjoints of
                                the policy, which are nearly all of the tape, are held for K steps at a
                                time and recomputed segment by segment in the backward sweep from the kept
                                states; the states and the Jacobians of the sample evaluation
                                (d_s + d_s (d_s + d_a) floats per trajectory and step) are kept for the
                                whole horizon.  Results are identical.  The per-segment tapes exist
                                twice, and the backward pass of a gradient call uses a second stream
                                owned by the context beside the caller's (forked after the forward pass,
                                joined before the call's last kernel is ordered on the caller's stream):
                                the replay of one segment and the weight gradient of another run beside
                                the sweep of a third. */
    int32_t cost_kind;       /* 0 quadratic tracking cost, 1 negative saturating reward of eq. (8) */
    float sigma_r;           /* width of eq. (8); used only if cost_kind == 1 */
} bagel_dims;

/* Number of policy parameters P for these dims, or BAGEL_EINVAL. */
int bagel_num_params(const bagel_dims *dims);

/*
 * Create a context for fixed dims on the current HIP device.  Allocates every buffer the rollout
 * calls, bagel_set_samples, bagel_sample_eval, bagel_adam_step and bagel_optimize need (model copy,
 * tape, partial sums); those calls allocate nothing.  The set-up calls allocate on their own:
 * bagel_prepare_samples, bagel_prepare_posterior and bagel_hyper_* share one float64 work space and up to
 * three internal streams, which the first of them makes, a later one enlarges if it needs more, and the
 * context keeps until bagel_destroy (so a loop over set-up calls allocates in its first pass only); the
 * first bagel_prepare_posterior also allocates the posterior cache, which the context keeps as well
 * (sizes at their declarations; bagel_workspace_bytes counts all of it).  `hip_stream` is a hipStream_t (NULL = default stream); all later work of this
 * context is enqueued there.
 * Errors: EINVAL (bad dims, null pointers), ENOMEM, EHIP.
 */
int bagel_create(bagel_ctx **out, const bagel_dims *dims, void *hip_stream);

/* Free everything the context owns (synchronises its stream first).  NULL is allowed. */
int bagel_destroy(bagel_ctx *ctx);

/* Device bytes held by the context. */
int64_t bagel_workspace_bytes(const bagel_ctx *ctx);

/*
 * Sample-set precompute (the one-time step before the rollouts; the pathwise counterpart of the
 * paper's one-time cache, Sec. IV-A).  For every output m: builds K_m + noise_var[m] I and Phi_m
 * in float64, factors it (Cholesky), solves for every sample, rounds v to float32, and installs
 * the model and samples in the context.
 *   X[N][D]  y[M][N]  lengthscale[M][D]  signal_var[M]  noise_var[M]
 *   omega[M][L][D] (already divided by the length scales)  phase[M][L]
 *   w[S][M][L]  eps[S][M][N]      (M = d_s)
 *   v_out[S][M][N] or NULL: receives the float32 representer weights.
 * Synchronises the stream (it must learn whether the factorisation succeeded).  Set-up work: it
 * needs 8 (Np^2 + Np L + Np S + S L) bytes of the set-up work space (see bagel_create) for each of up
 * to three outputs that it works on side by side on internal streams (ordered after what is already
 * enqueued on the context's stream; all finished on return; fewer side by side if the memory for three
 * cannot be had).
 * Errors: EINVAL, ENOMEM, ENOTPD (context is left unprepared), EHIP.
 */
int bagel_prepare_samples(bagel_ctx *ctx, const float *X, const float *y, const float *lengthscale,
                          const float *signal_var, const float *noise_var, const float *omega,
                          const float *phase, const float *w, const float *eps, float *v_out);

/*
 * Install a model with representer weights v[S][M][N] computed elsewhere (same arrays as
 * above otherwise; y and eps are not needed).  Lets a caller reuse stored samples, and lets
 * the tests drive the rollouts from exactly the float32 v the reference implementation used.
 * Errors: EINVAL, EHIP.
 */
int bagel_set_samples(bagel_ctx *ctx, const float *X, const float *lengthscale, const float *signal_var,
                      const float *omega, const float *phase, const float *w, const float *v);

/*
 * Forward pass and loss (Algorithm 1, forward pass).
 *   theta[P]  s0[B][d_s]  goals[H][B][d_g] (goals[t] is what the policy sees at step t and what
 *   the cost at s_{t+1} is measured against)
 *   loss[1]; loss_per_traj[B] or NULL (sum over t, not divided by B);
 *   states[H+1][B][d_s] or NULL.
 * Errors: EINVAL, ENOTPREPARED, EHIP.
 */
int bagel_rollout_loss(bagel_ctx *ctx, const float *theta, const float *s0, const float *goals,
                       float *loss, float *loss_per_traj, float *states);

/*
 * Forward pass, loss and backward pass (Algorithm 1: loss and its gradient with respect to
 * theta, here by a hand-written adjoint instead of automatic differentiation).
 *   grad_theta[P] (same layout as theta); grad_s0[B][d_s] or NULL (d loss / d s0);
 *   other arguments as in bagel_rollout_loss.
 * The result does not depend on ckpt_interval.  Errors: EINVAL, ENOTPREPARED, EHIP.
 */
int bagel_rollout_loss_grad(bagel_ctx *ctx, const float *theta, const float *s0, const float *goals,
                            float *loss, float *grad_theta, float *loss_per_traj, float *states,
                            float *grad_s0);

/*
 * Per-step posterior sampler: Algorithm 1 as printed draws the next state at every step from the
 * predictive posterior (eq. (9)) with the moments of eq. (2) (zero prior mean) and eq. (3), one
 * independent GP per state.  Here the draw is reparameterised with standard normal numbers the
 * caller supplies, f_m = mu_m(x) + sqrt(var_m(x)) xi, and the moments are exact (K_hat^-1 is kept;
 * the Lanczos variance estimates the paper uses are an approximation of the same quantity and are not
 * part of this library).  Cost per trajectory, step and output: 2 N^2 flop in float64, so this
 * sampler is meant for N of a few thousand; the pathwise calls above cost 2 N (D+1).
 *
 * bagel_prepare_posterior: alpha_m = K_hat_m^-1 y_m and K_hat_m^-1 for every output, float64, kept in
 * the context (the first call allocates 8 M (Np^2 + Np B (1 + (1+D)/32)) bytes, Np = N rounded up to 64:
 * K_hat^-1, the kernel rows of a step and the per-tile sums of its moments).
 * Arrays as in bagel_prepare_samples.  Synchronises the stream.  Errors: EINVAL, ENOMEM, ENOTPD, EHIP.
 *
 * bagel_posterior_rollout_loss / _grad: as bagel_rollout_loss / bagel_rollout_loss_grad, with
 * xi[H][B][M] (M = d_s): the draw used for output m of trajectory b at step t.  A variance below
 * 1e-12 is held at 1e-12 and its derivative taken as zero.  Errors: EINVAL, ENOTPREPARED, EHIP.
 */
int bagel_prepare_posterior(bagel_ctx *ctx, const float *X, const float *y, const float *lengthscale,
                            const float *signal_var, const float *noise_var);
int bagel_posterior_rollout_loss(bagel_ctx *ctx, const float *theta, const float *s0, const float *goals,
                                 const float *xi, float *loss, float *loss_per_traj, float *states);
int bagel_posterior_rollout_loss_grad(bagel_ctx *ctx, const float *theta, const float *s0, const float *goals,
                                      const float *xi, float *loss, float *grad_theta, float *loss_per_traj,
                                      float *states, float *grad_s0);

/*
 * One Adam update of the policy parameters on the device (Sec. III-C: the parameters are updated
 * with Adam; Algorithm 1, "update theta via gradient descent").  step >= 1 is the update counter:
 *   m <- beta1 m + (1 - beta1) g;  v <- beta2 v + (1 - beta2) g^2;
 *   theta <- theta - lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps).
 * theta[P], adam_m[P], adam_v[P] are device arrays owned by the caller and updated in place
 * (start the moments at zero); grad[P] is read.  Stored in float32, arithmetic in float64.
 * The paper fixes lr = 1e-2 (Sec. IV-A); beta1 = 0.9, beta2 = 0.999, eps = 1e-8 are Adam's defaults.
 * Errors: EINVAL (null pointer, step < 1, betas outside [0, 1), lr or eps not positive), EHIP.
 */
int bagel_adam_step(bagel_ctx *ctx, float *theta, const float *grad, float *adam_m, float *adam_v,
                    int step, float lr, float beta1, float beta2, float eps);

/*
 * Inner loop of Algorithm 1 (forward pass, backward pass, parameter update), n_iters times,
 * enqueued on the context's stream without any host synchronisation.  Iteration i (0-based)
 * rolls out from s0_sets[i % n_sets] towards goal_sets[i % n_sets], writes its loss to
 * loss_history[i] and applies Adam update number first_step + i.
 *   s0_sets[n_sets][B][d_s], goal_sets[n_sets][H][B][d_g]: n_sets = 1 is the fixed start and goal of
 *   Sec. IV-A, several sets are batches of starts and goals drawn by the caller (Sec. IV-B); the
 *   library draws no random numbers.  theta, adam_m, adam_v as in bagel_adam_step; loss_history[n_iters].
 * The function samples stay as installed; to redraw them between iterations call the loop with
 * n_iters = 1 and bagel_prepare_samples in between (the optimiser state lives with the caller).
 * Errors: EINVAL, ENOTPREPARED, EHIP.
 */
int bagel_optimize(bagel_ctx *ctx, float *theta, float *adam_m, float *adam_v, const float *s0_sets,
                   const float *goal_sets, int n_sets, int n_iters, int first_step, float lr,
                   float beta1, float beta2, float eps, float *loss_history);

/*
 * GP hyper-parameter learning (Algorithm 1, "learn GP transition dynamics"): the log marginal
 * likelihood of eq. (5) for every output,
 *   lml_m = -1/2 y_m^T K_hat^-1 y_m - 1/2 log|K_hat| - N/2 log(2 pi),
 * and its gradient (eq. (6) in its standard form, 1/2 tr((a a^T - K_hat^-1) dK_hat/dphi), a = K_hat^-1 y)
 * with respect to the logarithms of the hyper-parameters of eq. (4):
 *   log_hyp[M][D+2] = (log l_1 .. log l_D, log alpha^2, log sigma_n^2) per output.
 * X[N][D], y[M][N] as in bagel_prepare_samples; lml[M]; grad[M][D+2] or NULL.  Float64 inside.
 * Set-up work: needs three Np x Np float64 matrices per output worked on (set-up work space, see
 * bagel_create) and synchronises the stream.
 * Errors: EINVAL, ENOMEM, ENOTPD, EHIP.
 *
 * bagel_hyper_fit: n_iters Adam updates of log_hyp (in place) that raise lml / N of every output;
 * adam_m, adam_v [M][D+2] are the caller's optimiser state (start at zero), first_step >= 1 the
 * number of the first update; lml_history[n_iters][M] receives the lml before each update.
 * The paper does not state the optimiser settings of this step; they are arguments.
 */
int bagel_hyper_lml_grad(bagel_ctx *ctx, const float *X, const float *y, const float *log_hyp, float *lml,
                         float *grad);
int bagel_hyper_fit(bagel_ctx *ctx, const float *X, const float *y, float *log_hyp, float *adam_m, float *adam_v,
                    int n_iters, int first_step, float lr, float beta1, float beta2, float eps,
                    float *lml_history);

/*
 * One evaluation of the function samples (the transition model alone): for every trajectory b,
 * f[b][m] = f_{s(b),m}(x[b]) and, if jac != NULL, jac[b][m][d] = d f / d x_d.   x[B][D].
 * Runs the same kernels as one rollout step.  Errors: EINVAL, ENOTPREPARED, EHIP.
 */
int bagel_sample_eval(bagel_ctx *ctx, const float *x, float *f, float *jac);

/*
 * bagel_sample_eval for callers that cannot allocate device memory or hold a context: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  One call does what
 * bagel_set_samples + bagel_sample_eval do (model re-layout, then f and optionally jac for every
 * trajectory, arrays as documented there: X[N][D] lengthscale[M][D] signal_var[M] omega[M][L][D]
 * phase[M][L] w[S][M][L] v[S][M][N] x[B][D] -> f[B][M], jac[B][M][D] or NULL; of dims only d_s, d_a,
 * N, L, S, B matter, the rest must merely be valid) with the same kernels, on `hip_stream`, but keeps
 * every intermediate buffer in one static device array of BAGEL_STATIC_SCRATCH_BYTES that the library
 * holds on each GPU it runs on until the process ends.  It calls no hipMalloc, hipFree or other
 * allocating routine, creates no context and does not synchronise.  The first call on a device looks
 * up the array's address (hipGetSymbolAddress); make that call outside a capture.
 * Size limit: 8 M (Np + Lp) (D+1) + 4 M (Np + Lp) S + 8 B (D + M + groups (1+D)) bytes plus alignment
 * must fit the array (Np, Lp: N, L rounded up to the work-unit size, groups <= M (N + L) / 128 + 2 M);
 * e.g. N = 512, L = 1024, S = B = 256, D = 5 needs 7 MB.  Larger sizes are rejected with EINVAL.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different
 * streams or threads) race; calls on one stream are safe, and a call never reads what an earlier call
 * left in the array.  Errors: EINVAL, EHIP; message through bagel_last_error(NULL).
 */
#define BAGEL_STATIC_SCRATCH_BYTES (32u << 20)
int bagel_sample_eval_static(const bagel_dims *dims, void *hip_stream, const float *X, const float *lengthscale,
                             const float *signal_var, const float *omega, const float *phase, const float *w,
                             const float *v, const float *x, float *f, float *jac);

/*
 * Measurement hooks (used by bench.py; not part of the method).  With every > 0, every
 * `every`-th launch of the sample-evaluation kernel inside the rollout calls (for the posterior
 * sampler: the launches of one step, all outputs) is bracketed by
 * HIP events on the context's stream (at most 4096 timed launches between two reads; further
 * ones are skipped).  bagel_profile_read synchronises the stream, returns the summed elapsed
 * milliseconds and the number of timed launches since the last read, and resets both.
 * Errors: EINVAL, EHIP.
 */
int bagel_profile_enable(bagel_ctx *ctx, int every);
int bagel_profile_read(bagel_ctx *ctx, double *kernel_ms, int *launches);

/* Message of the last error on this context ("" if none); valid until the next call on it.
 * With ctx == NULL: message of the last failed bagel_create on this thread. */
const char *bagel_last_error(const bagel_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* BAGEL_H */
