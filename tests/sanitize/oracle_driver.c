/*
 * Host sanitizer driver for the CPU oracle: compiles oracle/bagel_oracle.c into this program with
 * -fsanitize=address,undefined and runs every exported function once on small, exactly sized heap
 * arrays (so that an access one element past an extent is an error), with odd sizes, shared samples
 * (S < B), two hidden layers, a bounded action and both cost kinds.  The numbers are checked
 * elsewhere (tests/test_oracle_pins.py); this run only has to finish without a sanitizer report.
 */
#include "../../oracle/bagel_oracle.c"

#include <stdio.h>

static double *fill(size_t n, unsigned *seed, double scale)
{
    double *p = (double *)malloc((n ? n : 1) * sizeof(double));
    for (size_t i = 0; i < n; ++i) {
        *seed = *seed * 1664525u + 1013904223u;
        p[i] = scale * ((double)(*seed >> 8) / 8388608.0 - 1.0);
    }
    return p;
}

static int run_case(int cost_kind, double act_bound, int n_hidden)
{
    oracle_dims dm;
    memset(&dm, 0, sizeof(dm));
    dm.d_s = 3; dm.d_a = 2; dm.d_g = 2;
    dm.N = 13; dm.L = 7; dm.S = 3; dm.B = 6; dm.H = 5;
    dm.n_hidden = n_hidden; dm.hidden[0] = 5; dm.hidden[1] = 4;
    dm.act_bound = act_bound;
    dm.tracked[0] = 2; dm.tracked[1] = 0; dm.q[0] = 1.0; dm.q[1] = 0.5;
    dm.cost_kind = cost_kind; dm.sigma_r = 0.7;
    const int D = dm.d_s + dm.d_a, M = dm.d_s, N = dm.N, L = dm.L, S = dm.S, B = dm.B, H = dm.H;
    const int P = oracle_num_params(&dm);
    unsigned seed = 12345u + (unsigned)cost_kind;
    double *X = fill((size_t)N * D, &seed, 1.0), *y = fill((size_t)M * N, &seed, 0.1);
    double *ell = fill((size_t)M * D, &seed, 0.4), *sf2 = fill(M, &seed, 0.2), *sn2 = fill(M, &seed, 0.0);
    for (int i = 0; i < M * D; ++i) ell[i] = 1.0 + ell[i];
    for (int i = 0; i < M; ++i) { sf2[i] = 0.8 + sf2[i]; sn2[i] = 1e-3; }
    double *omega = fill((size_t)M * L * D, &seed, 1.0), *phase = fill((size_t)M * L, &seed, 3.0);
    double *w = fill((size_t)S * M * L, &seed, 1.0), *eps = fill((size_t)S * M * N, &seed, 0.03);
    double *v = fill((size_t)S * M * N, &seed, 0.0);
    double *theta = fill((size_t)P, &seed, 0.3), *s0 = fill((size_t)B * dm.d_s, &seed, 0.5);
    double *goals = fill((size_t)H * B * dm.d_g, &seed, 1.0);
    int rc = oracle_prepare_samples(&dm, X, y, ell, sf2, sn2, omega, phase, w, eps, v);
    if (rc != 0) return 10 + rc;
    (void)oracle_kernel(D, ell, sf2[0], X, X + D);
    double *phi = fill((size_t)L, &seed, 0.0);
    oracle_features(D, L, sf2[1], omega + (size_t)L * D, phase + L, X, phi);
    double *f = fill((size_t)M, &seed, 0.0), *J = fill((size_t)M * D, &seed, 0.0);
    oracle_sample_eval(&dm, X, ell, sf2, omega, phase, w + (size_t)(S - 1) * M * L, v + (size_t)(S - 1) * M * N,
                       X + (size_t)(N - 1) * D, f, J);
    oracle_sample_eval(&dm, X, ell, sf2, omega, phase, w, v, X, f, NULL);
    double *h0 = fill((size_t)(dm.d_s + dm.d_g), &seed, 1.0), *act = fill((size_t)dm.d_a, &seed, 0.0);
    oracle_policy(&dm, theta, h0, act);
    double loss, *lpt = fill((size_t)B, &seed, 0.0), *states = fill((size_t)(H + 1) * B * dm.d_s, &seed, 0.0);
    double *gth = fill((size_t)P, &seed, 0.0), *gs0 = fill((size_t)B * dm.d_s, &seed, 0.0);
    rc = oracle_rollout(&dm, X, ell, sf2, omega, phase, w, v, theta, s0, goals, &loss, lpt, states, gth, gs0);
    if (rc != 0 || !(loss == loss)) return 20;
    rc = oracle_rollout(&dm, X, ell, sf2, omega, phase, w, v, theta, s0, goals, &loss, NULL, NULL, NULL, NULL);
    if (rc != 0) return 21;
    double *alpha = fill((size_t)M * N, &seed, 0.0), *Kinv = fill((size_t)M * N * N, &seed, 0.0);
    rc = oracle_posterior_prepare(&dm, X, y, ell, sf2, sn2, alpha, Kinv);
    if (rc != 0) return 30;
    double mu[8], var[8], *dmu = fill((size_t)M * D, &seed, 0.0), *dvar = fill((size_t)M * D, &seed, 0.0);
    double *work = fill((size_t)2 * N, &seed, 0.0);
    oracle_posterior_moments(&dm, X, ell, sf2, alpha, Kinv, X + D, mu, var, dmu, dvar, work);
    double *xi = fill((size_t)H * B * M, &seed, 1.0);
    rc = oracle_posterior_rollout(&dm, X, ell, sf2, alpha, Kinv, xi, theta, s0, goals, &loss, lpt, states, gth, gs0);
    if (rc != 0 || !(loss == loss)) return 40;
    double *am = fill((size_t)P, &seed, 0.0), *av = fill((size_t)P, &seed, 0.0);
    oracle_adam_step(P, theta, gth, am, av, 1, 1e-2, 0.9, 0.999, 1e-8);
    /* a factorisation that must fail cleanly: negative noise on duplicated points */
    memcpy(X + D, X, (size_t)D * sizeof(double));
    sn2[0] = -1.0;
    rc = oracle_prepare_samples(&dm, X, y, ell, sf2, sn2, omega, phase, w, eps, v);
    if (rc == 0) return 50;
    double *all[] = {X, y, ell, sf2, sn2, omega, phase, w, eps, v, theta, s0, goals, phi, f, J, h0, act, lpt, states,
                     gth, gs0, alpha, Kinv, dmu, dvar, work, xi, am, av};
    for (size_t i = 0; i < sizeof(all) / sizeof(all[0]); ++i) free(all[i]);
    return 0;
}

int main(void)
{
    int rc = run_case(0, 0.0, 1);
    if (rc == 0) rc = run_case(1, 1.5, 2);
    printf("oracle sanitizer driver: %s (%d), %d threads\n", rc == 0 ? "ok" : "FAILED", rc, oracle_num_threads());
    return rc;
}
