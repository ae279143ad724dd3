/*
 * CPU oracle (float64, plain loops) for batched Monte-Carlo policy rollouts
 * through pathwise-sampled Gaussian-process dynamics and the reverse-mode
 * gradient of the mean trajectory cost with respect to the policy parameters.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the HIP implementation and
 * to be timed beside it as a CPU baseline.  It shares no code, header, table
 * or helper with the HIP path, and the product never calls it.
 *
 * What each function follows in the paper (arXiv 2202.13638):
 *   oracle_kernel           Sec. III-A, eq. (4): squared-exponential ARD kernel,
 *                           Lambda read as diag(1 / l_d^2).
 *   oracle_features         random Fourier features of that kernel (the prior
 *                           part of a pathwise sample; Sec. II cites pathwise
 *                           conditioning as the batch-rollout sampler).
 *   oracle_prepare_samples  Sec. III-A: K_hat = K + sigma_n^2 I as below eq. (3);
 *                           Matheron update v = K_hat^{-1} (y - Phi w - eps).
 *   oracle_sample_eval      one function sample f(x) = phi(x)^T w + k(x,X)^T v
 *                           and its Jacobian with respect to x.
 *   oracle_rollout          Algorithm 1, forward pass (policy, sampled
 *                           transition on state differences as in Sec. III-A,
 *                           running cost) and loss = (1/b) * sum as in eq. (10),
 *                           (11); backward pass = the adjoint of exactly those
 *                           steps, summed over trajectories and time.
 *   oracle_posterior_*      the sampler of Algorithm 1 as printed: at every step the next
 *                           state is drawn from the predictive posterior, eq. (9), with the
 *                           moments of eq. (2) (zero prior mean) and eq. (3), one independent
 *                           GP per state (Sec. III-A).  The draw is reparameterised,
 *                           f = mu(x) + sqrt(var(x)) * xi with xi ~ N(0,1) handed in, so that
 *                           the loss is differentiable in theta (Sec. III-B differentiates
 *                           through the sampled transitions).  Exact moments from K_hat^-1;
 *                           the Lanczos variance estimates the paper uses to speed this up are
 *                           an approximation of the same quantity and are not reproduced.
 *   oracle_adam_step        Algorithm 1, the parameter update: Sec. III-C names
 *                           Adam (Kingma & Ba) as the gradient-descent rule; the
 *                           update is that paper's Algorithm 1 with bias-corrected
 *                           moment estimates.  The inner loop of Algorithm 1
 *                           (oracle.optimize in the Python wrapper) alternates
 *                           oracle_rollout and oracle_adam_step.
 *
 * (GP hyper-parameter learning by the marginal likelihood, eq. (5), (6), is the plain numpy
 * function hyper_lml_grad in the Python wrapper; pinned against scikit-learn and finite differences.)
 *
 * Pins (tests/test_oracle_pins.py): with w = 0 and eps = 0 a sample is the
 * textbook posterior mean of eq. (2); sample mean / covariance over many draws
 * against eq. (2), (3); feature inner products against eq. (4); central finite
 * differences and an independent autodiff graph for the gradient; H = 1 closed
 * form; additivity over trajectories; the Adam step against its closed form for a
 * constant gradient and against torch.optim.Adam; the posterior moments against scipy's
 * Cholesky solve, the N = 1 closed form, finite differences, and (xi = 0) the pathwise rollout
 * with a zero draw.  The numerical values of a rollout on the
 * synthetic workloads themselves are not printed anywhere in the paper.
 *
 * Conventions: row-major arrays; X[N][D]; per output m: ell[M][D], sf2[M]
 * (alpha^2), sn2[M] (sigma_n^2), omega[M][L][D] (already divided by the
 * length scales), phase[M][L]; per sample s: w[S][M][L], eps[S][M][N],
 * v[S][M][N].  theta: for each layer W[out][in] then b[out].
 * Trajectory b uses sample b / (B / S).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t d_s, d_a, d_g;
    int32_t N, L, S, B, H;
    int32_t n_hidden;
    int32_t hidden[2];
    double act_bound;      /* <= 0: linear output; > 0: a = act_bound * tanh(z) */
    int32_t tracked[8];    /* state index of each goal component */
    double q[8];           /* cost weights */
    int32_t cost_kind;     /* 0: quadratic cost sum_j q_j (s_ij - g_j)^2 ;
                              1: negative saturating reward of eq. (8):
                                 -exp(-(1/(2 sigma_r^2)) sum_j q_j (s_ij - g_j)^2) */
    double sigma_r;
} oracle_dims;

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* eq. (4) with Lambda = diag(1/l_d^2) */
double oracle_kernel(int D, const double *ell, double sf2, const double *xa, const double *xb)
{
    double r = 0.0;
    for (int d = 0; d < D; ++d) {
        double t = (xa[d] - xb[d]) / ell[d];
        r += t * t;
    }
    return sf2 * exp(-0.5 * r);
}

/* phi(x)_l = sqrt(2 alpha^2 / L) cos(omega_l . x + phase_l) */
void oracle_features(int D, int L, double sf2, const double *omega, const double *phase,
                     const double *x, double *phi_out)
{
    double amp = sqrt(2.0 * sf2 / (double)L);
    for (int l = 0; l < L; ++l) {
        double z = phase[l];
        for (int d = 0; d < D; ++d) z += omega[(size_t)l * D + d] * x[d];
        phi_out[l] = amp * cos(z);
    }
}

/* Lower Cholesky factor in place (column by column); returns -1 on a pivot <= 0. */
static int cholesky_lower(double *A, int n)
{
    for (int j = 0; j < n; ++j) {
        double *Aj = A + (size_t)j * n;
        double d = Aj[j];
        for (int k = 0; k < j; ++k) d -= Aj[k] * Aj[k];
        if (!(d > 0.0)) return -1;
        d = sqrt(d);
        Aj[j] = d;
#pragma omp parallel for schedule(static)
        for (int i = j + 1; i < n; ++i) {
            double *Ai = A + (size_t)i * n;
            double s = Ai[j];
            for (int k = 0; k < j; ++k) s -= Ai[k] * Aj[k];
            Ai[j] = s / d;
        }
    }
    return 0;
}

/* solve L L^T x = b in place, L lower (row-major, leading dimension n) */
static void cholesky_solve(const double *Lm, int n, double *b)
{
    for (int i = 0; i < n; ++i) {
        const double *Li = Lm + (size_t)i * n;
        double s = b[i];
        for (int k = 0; k < i; ++k) s -= Li[k] * b[k];
        b[i] = s / Li[i];
    }
    for (int i = n - 1; i >= 0; --i) {
        double s = b[i];
        for (int k = i + 1; k < n; ++k) s -= Lm[(size_t)k * n + i] * b[k];
        b[i] = s / Lm[(size_t)i * n + i];
    }
}

/*
 * v[s][m][:] = (K_m + sn2_m I)^{-1} (y_m - Phi_m w_sm - eps_sm)   for every sample s and output m.
 * Returns 0, or -(m+1) if the Cholesky factorisation of output m hit a non-positive pivot.
 */
int oracle_prepare_samples(const oracle_dims *dm, const double *X, const double *y,
                           const double *ell, const double *sf2, const double *sn2,
                           const double *omega, const double *phase,
                           const double *w, const double *eps, double *v_out)
{
    const int D = dm->d_s + dm->d_a, M = dm->d_s, N = dm->N, L = dm->L, S = dm->S;
    double *K = (double *)malloc((size_t)N * N * sizeof(double));
    double *Phi = (double *)malloc((size_t)N * L * sizeof(double));
    if (!K || !Phi) { free(K); free(Phi); return -1000; }
    int rc = 0;
    for (int m = 0; m < M && rc == 0; ++m) {
        const double *ell_m = ell + (size_t)m * D;
        const double *om_m = omega + (size_t)m * L * D;
        const double *ph_m = phase + (size_t)m * L;
#pragma omp parallel for schedule(static)
        for (int i = 0; i < N; ++i) {
            for (int j = 0; j < N; ++j)
                K[(size_t)i * N + j] = oracle_kernel(D, ell_m, sf2[m], X + (size_t)i * D, X + (size_t)j * D);
            K[(size_t)i * N + i] += sn2[m];
            oracle_features(D, L, sf2[m], om_m, ph_m, X + (size_t)i * D, Phi + (size_t)i * L);
        }
        if (cholesky_lower(K, N) != 0) { rc = -(m + 1); break; }
#pragma omp parallel for schedule(static)
        for (int s = 0; s < S; ++s) {
            const double *w_sm = w + ((size_t)s * M + m) * L;
            const double *e_sm = eps + ((size_t)s * M + m) * N;
            double *v_sm = v_out + ((size_t)s * M + m) * N;
            for (int i = 0; i < N; ++i) {
                double prior = 0.0;
                for (int l = 0; l < L; ++l) prior += Phi[(size_t)i * L + l] * w_sm[l];
                v_sm[i] = y[(size_t)m * N + i] - prior - e_sm[i];
            }
            cholesky_solve(K, N, v_sm);
        }
    }
    free(K);
    free(Phi);
    return rc;
}

/*
 * One function sample at one input: f[m] = phi_m(x)^T w_m + k_m(x, X)^T v_m and, if J != NULL,
 * J[m][d] = d f[m] / d x[d].   w_s is [M][L], v_s is [M][N] (the rows of one sample).
 */
void oracle_sample_eval(const oracle_dims *dm, const double *X, const double *ell, const double *sf2,
                        const double *omega, const double *phase,
                        const double *w_s, const double *v_s, const double *x,
                        double *f, double *J)
{
    const int D = dm->d_s + dm->d_a, M = dm->d_s, N = dm->N, L = dm->L;
    for (int m = 0; m < M; ++m) {
        const double *ell_m = ell + (size_t)m * D;
        const double *om_m = omega + (size_t)m * L * D;
        const double *ph_m = phase + (size_t)m * L;
        const double amp = sqrt(2.0 * sf2[m] / (double)L);
        double val = 0.0;
        double g[16];
        for (int d = 0; d < D; ++d) g[d] = 0.0;
        /* prior part: random Fourier features */
        for (int l = 0; l < L; ++l) {
            double z = ph_m[l];
            for (int d = 0; d < D; ++d) z += om_m[(size_t)l * D + d] * x[d];
            double wl = w_s[(size_t)m * L + l];
            val += amp * cos(z) * wl;
            if (J) {
                double c = -amp * sin(z) * wl;
                for (int d = 0; d < D; ++d) g[d] += c * om_m[(size_t)l * D + d];
            }
        }
        /* update part: kernel row against the training inputs */
        for (int n = 0; n < N; ++n) {
            const double *Xn = X + (size_t)n * D;
            double k = oracle_kernel(D, ell_m, sf2[m], x, Xn);
            double vk = v_s[(size_t)m * N + n] * k;
            val += vk;
            if (J)
                for (int d = 0; d < D; ++d) g[d] -= vk * (x[d] - Xn[d]) / (ell_m[d] * ell_m[d]);
        }
        f[m] = val;
        if (J)
            for (int d = 0; d < D; ++d) J[(size_t)m * D + d] = g[d];
    }
}

/* ---- policy: tanh MLP, linear or saturating output (Sec. IV-A, IV-B) ---- */

static int n_layers(const oracle_dims *dm) { return dm->n_hidden + 1; }

static void layer_widths(const oracle_dims *dm, int *wd)
{
    wd[0] = dm->d_s + dm->d_g;
    for (int i = 0; i < dm->n_hidden; ++i) wd[i + 1] = dm->hidden[i];
    wd[dm->n_hidden + 1] = dm->d_a;
}

int oracle_num_params(const oracle_dims *dm)
{
    int wd[4];
    layer_widths(dm, wd);
    int P = 0;
    for (int i = 0; i < n_layers(dm); ++i) P += wd[i + 1] * wd[i] + wd[i + 1];
    return P;
}

/*
 * act: concatenated activations h_0 (input), h_1, ..., h_{n_hidden}, then the pre-activation z_out
 * of the output layer; a: action.  Returns nothing; sizes follow layer_widths().
 */
static void policy_forward(const oracle_dims *dm, const double *theta, const double *h0,
                           double *act, double *a)
{
    int wd[4];
    layer_widths(dm, wd);
    const int nl = n_layers(dm);
    double *hin = act;
    for (int i = 0; i < wd[0]; ++i) hin[i] = h0[i];
    const double *p = theta;
    for (int l = 0; l < nl; ++l) {
        const int ni = wd[l], no = wd[l + 1];
        const double *W = p, *bias = p + (size_t)no * ni;
        double *hout = hin + ni;
        for (int o = 0; o < no; ++o) {
            double z = bias[o];
            for (int i = 0; i < ni; ++i) z += W[(size_t)o * ni + i] * hin[i];
            hout[o] = (l < nl - 1) ? tanh(z) : z;
        }
        p += (size_t)no * ni + no;
        hin = hout;
    }
    for (int o = 0; o < dm->d_a; ++o)
        a[o] = dm->act_bound > 0.0 ? dm->act_bound * tanh(hin[o]) : hin[o];
}

void oracle_policy(const oracle_dims *dm, const double *theta, const double *h0, double *a)
{
    int wd[4];
    layer_widths(dm, wd);
    int act_sz = dm->d_a;
    for (int i = 0; i <= dm->n_hidden; ++i) act_sz += wd[i];
    double *act = (double *)malloc((size_t)act_sz * sizeof(double));
    if (!act) return;
    policy_forward(dm, theta, h0, act, a);
    free(act);
}

/* running cost at a state and its derivative with respect to the tracked entries */
static double step_cost(const oracle_dims *dm, const double *s, const double *g, double *dc_ds /* [d_s] or NULL */)
{
    double e = 0.0;
    for (int j = 0; j < dm->d_g; ++j) {
        double r = s[dm->tracked[j]] - g[j];
        e += dm->q[j] * r * r;
    }
    if (dm->cost_kind == 0) {
        if (dc_ds)
            for (int j = 0; j < dm->d_g; ++j)
                dc_ds[dm->tracked[j]] += 2.0 * dm->q[j] * (s[dm->tracked[j]] - g[j]);
        return e;
    }
    double c = -exp(-e / (2.0 * dm->sigma_r * dm->sigma_r));
    if (dc_ds)
        for (int j = 0; j < dm->d_g; ++j)
            dc_ds[dm->tracked[j]] += -c * dm->q[j] * (s[dm->tracked[j]] - g[j]) / (dm->sigma_r * dm->sigma_r);
    return c;
}

/* The sampled transition of one trajectory at one step: f[M] = sampled state increment at x[D]
 * and, if J != NULL, J[M][D] = d f / d x.  Two samplers implement it (pathwise function samples,
 * per-step posterior draws); the rollout below is the same for both. */
typedef struct transition {
    void (*eval)(const struct transition *self, int b, int t, const double *x, double *f, double *J);
} transition;

typedef struct {
    transition base;
    const oracle_dims *dm;
    const double *X, *ell, *sf2, *omega, *phase, *w, *v;
    int per_sample;
} pathwise_transition;

static void pathwise_eval(const transition *self, int b, int t, const double *x, double *f, double *J)
{
    const pathwise_transition *p = (const pathwise_transition *)self;
    const int M = p->dm->d_s, sidx = b / p->per_sample;
    (void)t;
    oracle_sample_eval(p->dm, p->X, p->ell, p->sf2, p->omega, p->phase, p->w + (size_t)sidx * M * p->dm->L,
                       p->v + (size_t)sidx * M * p->dm->N, x, f, J);
}

static int rollout_core(const oracle_dims *dm, const transition *tr, const double *theta, const double *s0,
                        const double *goals, double *loss, double *loss_per_traj, double *states,
                        double *grad_theta, double *grad_s0);

/*
 * Algorithm 1, forward and backward pass.
 *   s0[B][d_s], goals[H][B][d_g]; the cost at s_{t+1} uses goals[t] (the goal the policy saw).
 *   loss = (1/B) sum_b sum_{t=1..H} c(s_t).
 * Outputs (each may be NULL): loss[1], loss_per_traj[B] (not divided by B), states[H+1][B][d_s],
 * grad_theta[P], grad_s0[B][d_s].  The backward pass runs only if grad_theta or grad_s0 is given.
 */
int oracle_rollout(const oracle_dims *dm, const double *X, const double *ell, const double *sf2,
                   const double *omega, const double *phase, const double *w, const double *v,
                   const double *theta, const double *s0, const double *goals,
                   double *loss, double *loss_per_traj, double *states,
                   double *grad_theta, double *grad_s0)
{
    if (dm->S < 1 || dm->B % dm->S != 0) return -1;
    pathwise_transition p;
    p.base.eval = pathwise_eval;
    p.dm = dm; p.X = X; p.ell = ell; p.sf2 = sf2; p.omega = omega; p.phase = phase; p.w = w; p.v = v;
    p.per_sample = dm->B / dm->S;
    return rollout_core(dm, &p.base, theta, s0, goals, loss, loss_per_traj, states, grad_theta, grad_s0);
}

static int rollout_core(const oracle_dims *dm, const transition *tr, const double *theta, const double *s0,
                        const double *goals, double *loss, double *loss_per_traj, double *states,
                        double *grad_theta, double *grad_s0)
{
    const int ds = dm->d_s, da = dm->d_a, dg = dm->d_g, D = ds + da, M = ds;
    const int B = dm->B, H = dm->H;
    if (ds > 8 || dg > 8 || D > 16) return -1;
    const int P = oracle_num_params(dm);
    const int nl = n_layers(dm);
    int wd[4];
    layer_widths(dm, wd);
    int act_sz = dm->d_a;                       /* z_out */
    for (int i = 0; i <= dm->n_hidden; ++i) act_sz += wd[i];
    const int want_grad = (grad_theta != NULL) || (grad_s0 != NULL);
    const int nthreads = oracle_num_threads();
    double *gpart = NULL;
    if (grad_theta) {
        gpart = (double *)calloc((size_t)nthreads * P, sizeof(double));
        if (!gpart) return -2;
    }
    double *lpt = (double *)malloc((size_t)B * sizeof(double));
    if (!lpt) { free(gpart); return -2; }
    int err = 0;

#pragma omp parallel
    {
#ifdef _OPENMP
        const int tid = omp_get_thread_num();
#else
        const int tid = 0;
#endif
        double *mygrad = gpart ? gpart + (size_t)tid * P : NULL;
        /* per-trajectory tape */
        double *S_tape = (double *)malloc((size_t)(H + 1) * ds * sizeof(double));
        double *A_tape = (double *)malloc((size_t)H * act_sz * sizeof(double));
        double *J_tape = (double *)malloc((size_t)H * M * D * sizeof(double));
        double *delta = (double *)malloc((size_t)2 * (4096 + 16) * sizeof(double));
        if (!S_tape || !A_tape || !J_tape || !delta) {
#pragma omp atomic write
            err = -2;
        } else {
#pragma omp for schedule(static)
            for (int b = 0; b < B; ++b) {
                double x[16], f[8], a[8], h0[16];
                for (int i = 0; i < ds; ++i) S_tape[i] = s0[(size_t)b * ds + i];
                double total = 0.0;
                /* ---- forward pass ---- */
                for (int t = 0; t < H; ++t) {
                    const double *s = S_tape + (size_t)t * ds;
                    const double *g = goals + ((size_t)t * B + b) * dg;
                    for (int i = 0; i < ds; ++i) h0[i] = s[i];
                    for (int j = 0; j < dg; ++j) h0[ds + j] = g[j];
                    policy_forward(dm, theta, h0, A_tape + (size_t)t * act_sz, a);
                    for (int i = 0; i < ds; ++i) x[i] = s[i];
                    for (int i = 0; i < da; ++i) x[ds + i] = a[i];
                    tr->eval(tr, b, t, x, f, want_grad ? J_tape + (size_t)t * M * D : NULL);
                    double *sn = S_tape + (size_t)(t + 1) * ds;
                    for (int i = 0; i < ds; ++i) sn[i] = s[i] + f[i];
                    total += step_cost(dm, sn, g, NULL);
                }
                lpt[b] = total;
                if (states)
                    for (int t = 0; t <= H; ++t)
                        for (int i = 0; i < ds; ++i)
                            states[((size_t)t * B + b) * ds + i] = S_tape[(size_t)t * ds + i];
                if (!want_grad) continue;
                /* ---- backward pass: lam = d loss / d s_t, swept from t = H down to 0 ---- */
                double lam[8], u[16];
                for (int i = 0; i < ds; ++i) lam[i] = 0.0;
                step_cost(dm, S_tape + (size_t)H * ds, goals + ((size_t)(H - 1) * B + b) * dg, lam);
                for (int i = 0; i < ds; ++i) lam[i] /= (double)B;
                for (int t = H - 1; t >= 0; --t) {
                    const double *Jt = J_tape + (size_t)t * M * D;
                    const double *act = A_tape + (size_t)t * act_sz;
                    for (int d = 0; d < D; ++d) {
                        double acc = 0.0;
                        for (int m = 0; m < M; ++m) acc += Jt[(size_t)m * D + d] * lam[m];
                        u[d] = acc;
                    }
                    /* policy backward, top layer first */
                    double *dcur = delta, *dnext = delta + 4096 + 16;
                    {
                        int off = 0;
                        for (int i = 0; i <= dm->n_hidden; ++i) off += wd[i];
                        const double *zout = act + off;
                        for (int o = 0; o < da; ++o) {
                            double dz = u[ds + o];
                            if (dm->act_bound > 0.0) {
                                double th = tanh(zout[o]);
                                dz *= dm->act_bound * (1.0 - th * th);
                            }
                            dcur[o] = dz;
                        }
                    }
                    size_t poff = (size_t)P;
                    int hoff = 0;
                    for (int i = 0; i <= dm->n_hidden; ++i) hoff += wd[i];
                    for (int l = nl - 1; l >= 0; --l) {
                        const int ni = wd[l], no = wd[l + 1];
                        poff -= (size_t)no * ni + no;
                        hoff -= ni;
                        const double *W = theta + poff;
                        const double *hin = act + hoff;
                        if (mygrad) {
                            double *gW = mygrad + poff, *gb = mygrad + poff + (size_t)no * ni;
                            for (int o = 0; o < no; ++o) {
                                for (int i = 0; i < ni; ++i) gW[(size_t)o * ni + i] += dcur[o] * hin[i];
                                gb[o] += dcur[o];
                            }
                        }
                        for (int i = 0; i < ni; ++i) {
                            double acc = 0.0;
                            for (int o = 0; o < no; ++o) acc += W[(size_t)o * ni + i] * dcur[o];
                            dnext[i] = (l > 0) ? acc * (1.0 - hin[i] * hin[i]) : acc;
                        }
                        double *tmp = dcur; dcur = dnext; dnext = tmp;
                    }
                    /* dcur now holds d loss / d h_0 = [d/ds ; d/dg] through the policy */
                    for (int i = 0; i < ds; ++i) lam[i] += u[i] + dcur[i];
                    if (t >= 1) {
                        double dc[8];
                        for (int i = 0; i < ds; ++i) dc[i] = 0.0;
                        step_cost(dm, S_tape + (size_t)t * ds, goals + ((size_t)(t - 1) * B + b) * dg, dc);
                        for (int i = 0; i < ds; ++i) lam[i] += dc[i] / (double)B;
                    }
                }
                if (grad_s0)
                    for (int i = 0; i < ds; ++i) grad_s0[(size_t)b * ds + i] = lam[i];
            }
        }
        free(S_tape); free(A_tape); free(J_tape); free(delta);
    }

    if (!err) {
        double tot = 0.0;
        for (int b = 0; b < B; ++b) tot += lpt[b];
        if (loss) *loss = tot / (double)B;
        if (loss_per_traj) memcpy(loss_per_traj, lpt, (size_t)B * sizeof(double));
        if (grad_theta) {
            for (int p = 0; p < P; ++p) {
                double acc = 0.0;
                for (int t = 0; t < nthreads; ++t) acc += gpart[(size_t)t * P + p];
                grad_theta[p] = acc;
            }
        }
    }
    free(gpart);
    free(lpt);
    return err;
}

/*
 * Exact GP posterior, eq. (2) and (3), per output m:
 *   alpha_m = K_hat_m^-1 y_m,   Kinv_m = K_hat_m^-1   (K_hat = K + sigma_n^2 I, kernel of eq. (4)).
 * alpha[M][N], Kinv[M][N][N].  Returns 0, or 1 + m if K_hat_m is not positive definite.
 */
int oracle_posterior_prepare(const oracle_dims *dm, const double *X, const double *y, const double *ell,
                             const double *sf2, const double *sn2, double *alpha, double *Kinv)
{
    const int N = dm->N, M = dm->d_s, D = dm->d_s + dm->d_a;
    double *K = (double *)malloc((size_t)N * N * sizeof(double));
    double *col = (double *)malloc((size_t)N * sizeof(double));
    if (!K || !col) { free(K); free(col); return -2; }
    int rc = 0;
    for (int m = 0; m < M && !rc; ++m) {
        for (int i = 0; i < N; ++i)
            for (int j = 0; j < N; ++j)
                K[(size_t)i * N + j] = oracle_kernel(D, ell + (size_t)m * D, sf2[m], X + (size_t)i * D, X + (size_t)j * D) +
                                       (i == j ? sn2[m] : 0.0);
        if (cholesky_lower(K, N)) { rc = 1 + m; break; }
        for (int i = 0; i < N; ++i) alpha[(size_t)m * N + i] = y[(size_t)m * N + i];
        cholesky_solve(K, N, alpha + (size_t)m * N);
        for (int j = 0; j < N; ++j) {                      /* column j of the inverse */
            for (int i = 0; i < N; ++i) col[i] = (i == j) ? 1.0 : 0.0;
            cholesky_solve(K, N, col);
            for (int i = 0; i < N; ++i) Kinv[((size_t)m * N + i) * N + j] = col[i];
        }
    }
    free(K); free(col);
    return rc;
}

#define ORACLE_VAR_FLOOR 1e-12   /* variance below this is held there (and its derivative is zero) */

/*
 * Posterior moments at x[D] for every output: mu[M] (eq. (2), zero prior mean), var[M] (eq. (3),
 * latent function: no observation noise added), and optionally their derivatives dmu[M][D],
 * dvar[M][D] with respect to x.  work: 2 N doubles.
 */
void oracle_posterior_moments(const oracle_dims *dm, const double *X, const double *ell, const double *sf2,
                              const double *alpha, const double *Kinv, const double *x, double *mu, double *var,
                              double *dmu, double *dvar, double *work)
{
    const int N = dm->N, M = dm->d_s, D = dm->d_s + dm->d_a;
    double *k = work, *q = work + N;
    for (int m = 0; m < M; ++m) {
        const double *l = ell + (size_t)m * D;
        for (int n = 0; n < N; ++n) k[n] = oracle_kernel(D, l, sf2[m], x, X + (size_t)n * D);
        double mean = 0.0, quad = 0.0;
        for (int i = 0; i < N; ++i) {
            double acc = 0.0;
            const double *row = Kinv + ((size_t)m * N + i) * N;
            for (int j = 0; j < N; ++j) acc += row[j] * k[j];
            q[i] = acc;
            mean += alpha[(size_t)m * N + i] * k[i];
            quad += k[i] * acc;
        }
        mu[m] = mean;
        double vv = sf2[m] - quad;                     /* k(x,x) = alpha^2 */
        const int floored = vv < ORACLE_VAR_FLOOR;
        var[m] = floored ? ORACLE_VAR_FLOOR : vv;
        if (dmu) {
            for (int d = 0; d < D; ++d) {
                double a = 0.0, b = 0.0;
                for (int n = 0; n < N; ++n) {
                    const double dk = k[n] * (X[(size_t)n * D + d] - x[d]) / (l[d] * l[d]);   /* d k_n / d x_d */
                    a += alpha[(size_t)m * N + n] * dk;
                    b += q[n] * dk;
                }
                dmu[(size_t)m * D + d] = a;
                dvar[(size_t)m * D + d] = floored ? 0.0 : -2.0 * b;
            }
        }
    }
}

typedef struct {
    transition base;
    const oracle_dims *dm;
    const double *X, *ell, *sf2, *alpha, *Kinv, *xi;     /* xi[H][B][M] standard normal draws */
} posterior_transition;

static void posterior_eval(const transition *self, int b, int t, const double *x, double *f, double *J)
{
    const posterior_transition *p = (const posterior_transition *)self;
    const int M = p->dm->d_s, D = p->dm->d_s + p->dm->d_a, N = p->dm->N;
    double mu[8], var[8], dmu[8 * 16], dvar[8 * 16];
    double *work = (double *)malloc((size_t)2 * N * sizeof(double));
    oracle_posterior_moments(p->dm, p->X, p->ell, p->sf2, p->alpha, p->Kinv, x, mu, var, J ? dmu : NULL, dvar, work);
    free(work);
    for (int m = 0; m < M; ++m) {
        const double z = p->xi[((size_t)t * p->dm->B + b) * M + m];
        const double sd = sqrt(var[m]);
        f[m] = mu[m] + sd * z;                          /* eq. (9), reparameterised */
        if (J)
            for (int d = 0; d < D; ++d) J[(size_t)m * D + d] = dmu[(size_t)m * D + d] + z * dvar[(size_t)m * D + d] / (2.0 * sd);
    }
}

/* Algorithm 1 with the per-step posterior sampler; arguments as oracle_rollout, xi[H][B][M]. */
int oracle_posterior_rollout(const oracle_dims *dm, const double *X, const double *ell, const double *sf2,
                             const double *alpha, const double *Kinv, const double *xi, const double *theta,
                             const double *s0, const double *goals, double *loss, double *loss_per_traj,
                             double *states, double *grad_theta, double *grad_s0)
{
    posterior_transition p;
    p.base.eval = posterior_eval;
    p.dm = dm; p.X = X; p.ell = ell; p.sf2 = sf2; p.alpha = alpha; p.Kinv = Kinv; p.xi = xi;
    return rollout_core(dm, &p.base, theta, s0, goals, loss, loss_per_traj, states, grad_theta, grad_s0);
}

/*
 * One Adam update (Sec. III-C: the policy parameters are updated with Adam), step counter t >= 1:
 *   m <- beta1 m + (1 - beta1) g;  v <- beta2 v + (1 - beta2) g^2;
 *   theta <- theta - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps).
 * theta, m, v are updated in place.
 */
void oracle_adam_step(int P, double *theta, const double *grad, double *m, double *v, int t,
                      double lr, double beta1, double beta2, double eps)
{
    const double c1 = 1.0 - pow(beta1, (double)t), c2 = 1.0 - pow(beta2, (double)t);
    for (int p = 0; p < P; ++p) {
        const double g = grad[p];
        m[p] = beta1 * m[p] + (1.0 - beta1) * g;
        v[p] = beta2 * v[p] + (1.0 - beta2) * g * g;
        const double mhat = m[p] / c1, vhat = v[p] / c2;
        theta[p] -= lr * mhat / (sqrt(vhat) + eps);
    }
}
