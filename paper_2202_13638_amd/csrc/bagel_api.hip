// C ABI of libbagel.so (declared in include/bagel.h): argument checks, the context and its
// buffers, and the per-call schedule of kernels.  A rollout is a host loop over the horizon that
// enqueues, per step, the sample evaluation (pathwise function samples, or the per-step posterior
// draw) and the end-of-step kernel, which also runs the policy of the next step, on the context's
// stream (Algorithm 1, forward pass); the gradient call then sweeps the tape backwards in one launch
// per tape segment (Algorithm 1, backward pass) and finishes with one weight-gradient GEMM per layer.
// bagel_optimize wraps that in the inner loop of Algorithm 1 with an Adam update per iteration.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>

#include "bagel_internal.h"

static thread_local char g_create_err[512] = "";

#define CREATE_FAIL(code, ...)                                    \
    do {                                                          \
        snprintf(g_create_err, sizeof(g_create_err), __VA_ARGS__); \
        return (code);                                            \
    } while (0)

static const char *check_dims(const bagel_dims *d)
{
    if (d->d_s < 1 || d->d_s > BAGEL_MAX_STATE) return "d_s must be in 1..8";
    if (d->d_a < 1 || d->d_a > BAGEL_MAX_STATE) return "d_a must be in 1..8";
    if (d->d_g < 1 || d->d_g > BAGEL_MAX_STATE || d->d_g > d->d_s) return "d_g must be in 1..min(8, d_s)";
    if (d->N < 1 || d->L < 1 || d->S < 1 || d->B < 1 || d->H < 1) return "N, L, S, B, H must be positive";
    if (d->S > d->B || d->B % d->S != 0) return "S must divide B";
    if (d->n_hidden < 1 || d->n_hidden > 2) return "n_hidden must be 1 or 2";
    for (int i = 0; i < d->n_hidden; ++i)
        if (d->hidden[i] < 1 || d->hidden[i] > BAGEL_MAX_HIDDEN) return "hidden width must be in 1..256";
    for (int j = 0; j < d->d_g; ++j)
        if (d->tracked[j] < 0 || d->tracked[j] >= d->d_s) return "tracked index out of range";
    if (d->ckpt_interval < 0) return "ckpt_interval must be >= 0";
    if (d->cost_kind != 0 && d->cost_kind != 1) return "cost_kind must be 0 or 1";
    if (d->cost_kind == 1 && !(d->sigma_r > 0.0f)) return "sigma_r must be positive for cost_kind 1";
    if ((int64_t)d->B * d->H > ((int64_t)1 << 40)) return "B * H too large";
    return nullptr;
}

static void layer_layout(const bagel_dims *d, int *width, int *w_off, int *b_off, int *P)
{
    width[0] = d->d_s + d->d_g;
    for (int i = 0; i < d->n_hidden; ++i) width[i + 1] = d->hidden[i];
    width[d->n_hidden + 1] = d->d_a;
    int off = 0;
    for (int l = 0; l <= d->n_hidden; ++l) {
        w_off[l] = off;
        off += width[l + 1] * width[l];
        b_off[l] = off;
        off += width[l + 1];
    }
    *P = off;
}

extern "C" int bagel_num_params(const bagel_dims *dims)
{
    if (!dims || check_dims(dims)) return BAGEL_EINVAL;
    int width[4], w_off[3], b_off[3], P;
    layer_layout(dims, width, w_off, b_off, &P);
    return P;
}

template <class T>
static hipError_t dev_alloc(bagel_ctx *c, T **p, size_t count)
{
    *p = nullptr;
    if (count == 0) count = 1;
    hipError_t e = hipMalloc((void **)p, count * sizeof(T));
    if (e == hipSuccess) c->bytes += (int64_t)(count * sizeof(T));
    return e;
}

static void free_all(bagel_ctx *c)
{
    void *ptrs[] = {c->Xs, c->Xn, c->near_ok, c->Os, c->Of, c->A, c->amp, c->exp_tab, c->v4, c->w4, c->xbuf, c->part, c->xbuf_alt, c->part_alt, c->lpt, c->lam,
                    c->tape_s, c->tape_J, c->tape_h_set[0][0], c->tape_h_set[0][1], c->tape_h_set[0][2], c->tape_a_set[0],
                    c->tape_d_set[0][0], c->tape_d_set[0][1], c->tape_d_set[0][2], c->tape_h_set[1][0], c->tape_h_set[1][1],
                    c->tape_h_set[1][2], c->tape_a_set[1], c->tape_d_set[1][0], c->tape_d_set[1][1], c->tape_d_set[1][2], c->wpad_f, c->wpad_b, c->gsplit, c->gacc, c->fbuf, c->gtheta, c->post_alpha, c->post_Kinv, c->post_Kx, c->post_sums};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
}

static void use_tape_set(bagel_ctx *c, int set)
{
    for (int l = 0; l < 3; ++l) {
        c->tape_h[l] = c->tape_h_set[set][l];
        c->tape_d[l] = c->tape_d_set[set][l];
    }
    c->tape_a = c->tape_a_set[set];
}

static void destroy_side(bagel_ctx *c)
{
    hipEvent_t *evs[] = {&c->ev_fork, &c->ev_join, &c->ev_replay[0], &c->ev_replay[1], &c->ev_sweep[0], &c->ev_sweep[1]};
    for (hipEvent_t *ev : evs)
        if (*ev) { (void)hipEventDestroy(*ev); *ev = nullptr; }
    if (c->side) { (void)hipStreamDestroy(c->side); c->side = nullptr; }
}

extern "C" int bagel_create(bagel_ctx **out, const bagel_dims *dims, void *hip_stream)
{
    if (!out || !dims) CREATE_FAIL(BAGEL_EINVAL, "bagel_create: null argument");
    *out = nullptr;
    if (const char *msg = check_dims(dims)) CREATE_FAIL(BAGEL_EINVAL, "bagel_create: %s", msg);
    bagel_ctx *c = new (std::nothrow) bagel_ctx();
    if (!c) CREATE_FAIL(BAGEL_ENOMEM, "bagel_create: host allocation failed");
    memset(c, 0, sizeof(*c));
    c->dm = *dims;
    c->D = dims->d_s + dims->d_a;
    c->M = dims->d_s;
    c->d_in = dims->d_s + dims->d_g;
    c->n_layers = dims->n_hidden + 1;
    layer_layout(dims, c->width, c->w_off, c->b_off, &c->P);
    c->stream = (hipStream_t)hip_stream;

    if (const char *msg = bagel_plan_sample_eval(c)) {     // msg is a string literal: it outlives c
        delete c;
        CREATE_FAIL(BAGEL_EINVAL, "bagel_create: %s", msg);
    }
    const int B = dims->B, M = c->M, D = c->D;

    const int K = dims->ckpt_interval;
    const int H = dims->H;
    c->T_tape = (K > 0 && K < H) ? K : H;
    c->ksplit = bagel_env_int("BAGEL_KSPLIT", 256);
    int wf_total = 0, wb_total = 0;
    for (int l = 0; l < c->n_layers; ++l) {
        const int no = c->width[l + 1], ni = c->width[l];
        c->wpf_off[l] = wf_total; c->wpf_rp[l] = (no + 31) / 32 * 32; c->wpf_kp[l] = (ni + 31) / 32 * 32;
        wf_total += c->wpf_rp[l] * c->wpf_kp[l];
        c->wpb_off[l] = wb_total; c->wpb_rp[l] = (ni + 31) / 32 * 32; c->wpb_kp[l] = (no + 31) / 32 * 32;
        wb_total += c->wpb_rp[l] * c->wpb_kp[l];
    }
    const size_t Bz = (size_t)B, T = (size_t)c->T_tape;

    hipError_t e = hipSuccess;
#define ALLOC(ptr, count)                         \
    if (e == hipSuccess) e = dev_alloc(c, &(ptr), (size_t)(count))
    ALLOC(c->Xs, (size_t)M * c->Np * (D + 1));
    ALLOC(c->Xn, (size_t)M * c->Np * (D + 1));
    ALLOC(c->near_ok, 1);
    ALLOC(c->Os, (size_t)M * c->Lp * (D + 1));
    ALLOC(c->Of, (size_t)M * c->Lp * 4 * ((D + 3) / 4));
    ALLOC(c->A, (size_t)M * D);
    ALLOC(c->amp, (size_t)M);
    ALLOC(c->exp_tab, 256);
    ALLOC(c->v4, (size_t)M * (c->Np / 4) * dims->S);
    ALLOC(c->w4, (size_t)M * (c->Lp / 4) * dims->S);
    ALLOC(c->xbuf, (size_t)D * Bz);
    ALLOC(c->part, (size_t)c->groups * (1 + D) * Bz);
    ALLOC(c->xbuf_alt, (size_t)D * Bz);
    ALLOC(c->part_alt, (size_t)c->groups * (1 + D) * Bz);
    ALLOC(c->lpt, Bz);
    ALLOC(c->lam, (size_t)dims->d_s * Bz);
    ALLOC(c->fbuf, (size_t)M * Bz);
    ALLOC(c->tape_s, (size_t)(H + 1) * dims->d_s * Bz);
    ALLOC(c->tape_J, (size_t)H * M * D * Bz);
    for (int set = 0; set < (c->T_tape < H ? 2 : 1); ++set) {
        for (int l = 0; l < c->n_layers; ++l) {
            // four rows of slack: the sweep reads its tanh outputs at a scalar row base (clamped to the layer)
            // plus a lane offset of up to four rows; what lies past the layer's rows is read but not used
            ALLOC(c->tape_h_set[set][l], (T * c->width[l] + 4) * Bz);
            ALLOC(c->tape_d_set[set][l], T * c->width[l + 1] * Bz);
        }
        ALLOC(c->tape_a_set[set], T * dims->d_a * Bz);
    }
    use_tape_set(c, 0);
    ALLOC(c->wpad_f, (size_t)wf_total);
    ALLOC(c->wpad_b, (size_t)wb_total);
    ALLOC(c->gsplit, (size_t)c->ksplit * c->P);
    ALLOC(c->gacc, (size_t)c->P);
    ALLOC(c->gtheta, (size_t)c->P);
#undef ALLOC
    if (e == hipSuccess) {
        // table of the sample-evaluation kernel's table form: -2^(i/256), high word lowered by i << 12
        uint64_t tab[256];
        for (int i = 0; i < 256; ++i) {
            const double t = exp2((double)i / 256.0);
            uint64_t bits;
            memcpy(&bits, &t, sizeof(bits));
            tab[i] = (bits | 0x8000000000000000ull) - ((uint64_t)i << 44);
        }
        e = hipMemcpy(c->exp_tab, tab, sizeof(tab), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess && c->T_tape < H) {
        // the side stream of the checkpointed backward pass (default priority) and the events that order it
        e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
        hipEvent_t *evs[] = {&c->ev_fork, &c->ev_join, &c->ev_replay[0], &c->ev_replay[1], &c->ev_sweep[0], &c->ev_sweep[1]};
        for (hipEvent_t *ev : evs)
            if (e == hipSuccess) e = hipEventCreateWithFlags(ev, hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        const int64_t want = c->bytes;
        destroy_side(c);
        free_all(c);
        delete c;
        (void)hipGetLastError();
        if (e == hipErrorOutOfMemory || e == hipErrorMemoryAllocation)
            CREATE_FAIL(BAGEL_ENOMEM, "bagel_create: device allocation failed after %lld bytes", (long long)want);
        CREATE_FAIL(BAGEL_EHIP, "bagel_create: hipMalloc failed: %s", hipGetErrorString(e));
    }
    g_create_err[0] = 0;
    *out = c;
    return BAGEL_OK;
}

extern "C" int bagel_destroy(bagel_ctx *c)
{
    if (!c) return BAGEL_OK;
    (void)hipStreamSynchronize(c->stream);
    if (c->prof_ev) {
        for (int i = 0; i < 2 * BAGEL_PROF_MAX; ++i)
            if (c->prof_ev[i]) (void)hipEventDestroy(c->prof_ev[i]);
        free(c->prof_ev);
    }
    bagel_release_setup(c);
    if (c->side) (void)hipStreamSynchronize(c->side);
    destroy_side(c);
    free_all(c);
    delete c;
    return BAGEL_OK;
}

extern "C" int64_t bagel_workspace_bytes(const bagel_ctx *c) { return c ? c->bytes : 0; }

extern "C" const char *bagel_last_error(const bagel_ctx *c) { return c ? c->err : g_create_err; }

extern "C" int bagel_set_samples(bagel_ctx *c, const float *X, const float *lengthscale, const float *signal_var,
                                 const float *omega, const float *phase, const float *w, const float *v)
{
    if (!c) return BAGEL_EINVAL;
    c->err[0] = 0;
    if (!X || !lengthscale || !signal_var || !omega || !phase || !w || !v)
        BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_set_samples: null argument");
    c->prepared = false;
    c->post_prepared = false;       // the model tables are shared: the posterior cache belongs to the old ones
    BAGEL_HIP(c, bagel_launch_build_model(c, X, lengthscale, signal_var, omega, phase));
    BAGEL_HIP(c, bagel_launch_pack_samples(c, w, v));
    c->prepared = true;
    return BAGEL_OK;
}

extern "C" int bagel_prepare_samples(bagel_ctx *c, const float *X, const float *y, const float *lengthscale,
                                     const float *signal_var, const float *noise_var, const float *omega,
                                     const float *phase, const float *w, const float *eps, float *v_out)
{
    if (!c) return BAGEL_EINVAL;
    c->err[0] = 0;
    if (!X || !y || !lengthscale || !signal_var || !noise_var || !omega || !phase || !w || !eps)
        BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_prepare_samples: null argument");
    c->prepared = false;
    c->post_prepared = false;       // the model tables are shared: the posterior cache belongs to the old ones
    BAGEL_HIP(c, bagel_launch_build_model(c, X, lengthscale, signal_var, omega, phase));
    BAGEL_HIP(c, bagel_launch_pack_samples(c, w, nullptr));
    const int rc = bagel_prepare_impl(c, X, y, lengthscale, signal_var, noise_var, omega, phase, w, eps, v_out);
    if (rc != BAGEL_OK) return rc;
    c->prepared = true;
    return BAGEL_OK;
}

static hipError_t gp_step_timed(bagel_ctx *c, bool jac, const float *xi_t = nullptr, float *prev_jac = nullptr);

extern "C" int bagel_sample_eval(bagel_ctx *c, const float *x, float *f, float *jac)
{
    if (!c) return BAGEL_EINVAL;
    c->err[0] = 0;
    if (!x || !f) BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_sample_eval: null argument");
    if (!c->prepared) BAGEL_FAIL(c, BAGEL_ENOTPREPARED, "bagel_sample_eval: no samples installed");
    BAGEL_HIP(c, bagel_launch_eval_io(c, 0, x, nullptr));
    BAGEL_HIP(c, gp_step_timed(c, jac != nullptr));
    BAGEL_HIP(c, bagel_launch_finalize(c, jac != nullptr, -1, jac));
    BAGEL_HIP(c, bagel_launch_eval_io(c, 1, nullptr, f));
    return BAGEL_OK;
}

// ---- sample evaluation without a context and without any allocation -------------------------------
// Everything bagel_sample_eval keeps in context-owned device buffers (the model in its internal layout,
// the re-laid-out sample streams, the inputs in float64, the partial sums of the work units, the
// summed values) lives here in one file-scope device array.  Every GPU the library runs on holds its
// own copy of the array at its own address until the process ends; host code may use the array only
// through the address hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[BAGEL_STATIC_SCRATCH_BYTES];

#define BAGEL_MAX_DEVICES 64
static std::mutex g_scratch_mutex;
static unsigned char *g_scratch_ptr[BAGEL_MAX_DEVICES];   // per device, resolved on the first call there

// device address of `scratch` on the current device (null and *err set on failure)
static unsigned char *scratch_base(hipError_t *err)
{
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= BAGEL_MAX_DEVICES) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    return g_scratch_ptr[dev];
}

// bytes of the static array a call with these dims uses, or BAGEL_EINVAL
static int64_t static_scratch_bytes(const bagel_dims *dims)
{
    if (!dims || check_dims(dims)) return BAGEL_EINVAL;
    bagel_ctx c;
    memset(&c, 0, sizeof(c));
    c.dm = *dims;
    c.D = dims->d_s + dims->d_a;
    c.M = dims->d_s;
    if (bagel_plan_sample_eval(&c)) return BAGEL_EINVAL;
    const int64_t M = c.M, D = c.D, B = dims->B, S = dims->S;
    const int64_t counts[] = {8 * M * c.Np * (D + 1), 8 * M * c.Lp * (D + 1), 16 * M * c.Lp * ((D + 3) / 4), 8 * M * D, 8 * M,
                              16 * M * (c.Np / 4) * S, 16 * M * (c.Lp / 4) * S, 8 * D * B,
                              8 * (int64_t)c.groups * (1 + D) * B, 8 * M * B};
    int64_t total = 0;
    for (int64_t n : counts) total += (n + 255) / 256 * 256;
    return total;
}

extern "C" int bagel_sample_eval_static(const bagel_dims *dims, void *hip_stream, const float *X,
                                        const float *lengthscale, const float *signal_var, const float *omega,
                                        const float *phase, const float *w, const float *v, const float *x, float *f,
                                        float *jac)
{
    if (!dims) CREATE_FAIL(BAGEL_EINVAL, "bagel_sample_eval_static: null argument");
    if (const char *msg = check_dims(dims)) CREATE_FAIL(BAGEL_EINVAL, "bagel_sample_eval_static: %s", msg);
    if (!X || !lengthscale || !signal_var || !omega || !phase || !w || !v || !x || !f)
        CREATE_FAIL(BAGEL_EINVAL, "bagel_sample_eval_static: null argument");
    const int64_t need = static_scratch_bytes(dims);
    if (need < 0) CREATE_FAIL(BAGEL_EINVAL, "bagel_sample_eval_static: too many work units for these sizes");
    if (need > (int64_t)BAGEL_STATIC_SCRATCH_BYTES)
        CREATE_FAIL(BAGEL_EINVAL, "bagel_sample_eval_static: these sizes need %lld bytes of scratch, the static buffer holds %lld",
                    (long long)need, (long long)BAGEL_STATIC_SCRATCH_BYTES);
    hipError_t e = hipSuccess;
    unsigned char *base = scratch_base(&e);
    if (!base) CREATE_FAIL(BAGEL_EHIP, "bagel_sample_eval_static: address of the static buffer: %s", hipGetErrorString(e));

    // a context on the host stack whose device pointers are carved out of the static array
    bagel_ctx c;
    memset(&c, 0, sizeof(c));
    c.dm = *dims;
    c.D = dims->d_s + dims->d_a;
    c.M = dims->d_s;
    c.stream = (hipStream_t)hip_stream;
    (void)bagel_plan_sample_eval(&c);             // cannot fail: static_scratch_bytes has planned the same dims
    c.exp_table = false;                    // the table form of exp2 reads a table this call does not have
    const size_t M = c.M, D = c.D, B = dims->B, S = dims->S;
    size_t off = 0;
    auto carve = [&](size_t bytes) {
        unsigned char *p = base + off;
        off += (bytes + 255) / 256 * 256;
        return p;
    };
    c.Xs = reinterpret_cast<double *>(carve(8 * M * c.Np * (D + 1)));
    c.Os = reinterpret_cast<double *>(carve(8 * M * c.Lp * (D + 1)));
    c.Of = reinterpret_cast<float *>(carve(16 * M * c.Lp * ((D + 3) / 4)));
    c.A = reinterpret_cast<double *>(carve(8 * M * D));
    c.amp = reinterpret_cast<double *>(carve(8 * M));
    c.v4 = reinterpret_cast<float4 *>(carve(16 * M * (c.Np / 4) * S));
    c.w4 = reinterpret_cast<float4 *>(carve(16 * M * (c.Lp / 4) * S));
    c.xbuf = reinterpret_cast<double *>(carve(8 * D * B));
    c.part = reinterpret_cast<double *>(carve(8 * (size_t)c.groups * (1 + D) * B));
    c.fbuf = reinterpret_cast<double *>(carve(8 * M * B));
    if ((int64_t)off != need) CREATE_FAIL(BAGEL_EINVAL, "bagel_sample_eval_static: internal size mismatch");

    // every byte a kernel below reads was written by a kernel before it in this call (padding rows
    // included), so nothing of an earlier call's contents is ever used and nothing needs clearing
#define STATIC_HIP(call)                                                                                  \
    do {                                                                                                  \
        hipError_t e__ = (call);                                                                          \
        if (e__ != hipSuccess)                                                                            \
            CREATE_FAIL(BAGEL_EHIP, "bagel_sample_eval_static: %s failed: %s", #call, hipGetErrorString(e__)); \
    } while (0)
    STATIC_HIP(bagel_launch_build_model(&c, X, lengthscale, signal_var, omega, phase));
    STATIC_HIP(bagel_launch_pack_samples(&c, w, v));
    STATIC_HIP(bagel_launch_eval_io(&c, 0, x, nullptr));
    STATIC_HIP(bagel_launch_gp_step(&c, jac != nullptr, nullptr));
    STATIC_HIP(bagel_launch_finalize(&c, jac != nullptr, -1, jac));
    STATIC_HIP(bagel_launch_eval_io(&c, 1, nullptr, f));
#undef STATIC_HIP
    g_create_err[0] = 0;
    return BAGEL_OK;
}

// the sample-evaluation launch (pathwise samples, or with xi_t the launches of one posterior step),
// optionally bracketed by events
static hipError_t gp_step_timed(bagel_ctx *c, bool jac, const float *xi_t, float *prev_jac)
{
    bool timed = false;
    if (c->prof_every > 0) {
        timed = (c->prof_seen++ % c->prof_every == 0) && c->prof_used < BAGEL_PROF_MAX;
        if (timed) {
            hipError_t e = hipEventRecord(c->prof_ev[2 * c->prof_used], c->stream);
            if (e != hipSuccess) return e;
        }
    }
    hipError_t e = xi_t ? bagel_launch_posterior_step(c, jac, xi_t) : bagel_launch_gp_step(c, jac, prev_jac);
    if (timed && e == hipSuccess) {
        e = hipEventRecord(c->prof_ev[2 * c->prof_used + 1], c->stream);
        c->prof_used++;
    }
    return e;
}

extern "C" int bagel_profile_enable(bagel_ctx *c, int every)
{
    if (!c || every < 0) return BAGEL_EINVAL;
    c->err[0] = 0;
    if (every > 0 && !c->prof_ev) {
        c->prof_ev = (hipEvent_t *)calloc(2 * BAGEL_PROF_MAX, sizeof(hipEvent_t));
        if (!c->prof_ev) BAGEL_FAIL(c, BAGEL_ENOMEM, "bagel_profile_enable: host allocation failed");
        for (int i = 0; i < 2 * BAGEL_PROF_MAX; ++i) BAGEL_HIP(c, hipEventCreate(&c->prof_ev[i]));
    }
    c->prof_every = every;
    c->prof_seen = 0;
    c->prof_used = 0;
    return BAGEL_OK;
}

extern "C" int bagel_profile_read(bagel_ctx *c, double *kernel_ms, int *launches)
{
    if (!c || !kernel_ms || !launches) return BAGEL_EINVAL;
    c->err[0] = 0;
    BAGEL_HIP(c, hipStreamSynchronize(c->stream));
    double total = 0.0;
    for (int i = 0; i < c->prof_used; ++i) {
        float ms = 0.0f;
        BAGEL_HIP(c, hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]));
        total += (double)ms;
    }
    *kernel_ms = total;
    *launches = c->prof_used;
    c->prof_used = 0;
    c->prof_seen = 0;
    return BAGEL_OK;
}

// Forward steps 0 .. H-1 from the state in xbuf and the policy input in tape slot 0.  jac: the sample
// evaluation also returns its Jacobian, kept in slot t of the Jacobian tape; acts: the policy's
// activations are kept in slot t of their tape (otherwise every step reuses slot 0).
// Only the value sums of a step are on the critical path (state, cost, next action); the Jacobian sums
// of the pathwise sampler, eight ninths of the partial sums with D = 8, feed nothing but the tape, so
// they are added up one step late, by extra workgroups inside the next step's sample evaluation (after
// the last step: by a launch of their own).  The two steps' inputs and sums live in buffers that swap.
static int run_forward(bagel_ctx *c, bool jac, bool acts, bool write_tape_s, const float *theta, const float *goals,
                       float *states_out)
{
    const int H = c->dm.H;
    const bool posterior = c->cur_xi != nullptr;
    const size_t jslot = (size_t)c->M * c->D * c->dm.B;
    for (int t = 0; t < H; ++t) {
        const int next_slot = t + 1 < H ? (acts ? t + 1 : 0) : -1;
        // the policy of the first step runs on its own; every later one is part of the previous step's tail
        if (t == 0) BAGEL_HIP(c, bagel_launch_policy_forward(c, 0, theta));
        float *prev_jac = (jac && !posterior && t > 0) ? c->tape_J + (size_t)(t - 1) * jslot : nullptr;
        BAGEL_HIP(c, gp_step_timed(c, jac, posterior ? c->cur_xi + (size_t)t * c->dm.B * c->M : nullptr, prev_jac));
        BAGEL_HIP(c, bagel_launch_step_tail(c, t, t, next_slot, jac, true, write_tape_s, theta, goals, states_out,
                                            posterior));
        double *tx = c->xbuf; c->xbuf = c->xbuf_alt; c->xbuf_alt = tx;
        double *tp = c->part; c->part = c->part_alt; c->part_alt = tp;
    }
    if (jac && !posterior) {
        // the last step's sums are in what is now the alternate pair
        double *tx = c->xbuf; c->xbuf = c->xbuf_alt; c->xbuf_alt = tx;
        double *tp = c->part; c->part = c->part_alt; c->part_alt = tp;
        BAGEL_HIP(c, bagel_launch_jac_reduce(c, c->tape_J + (size_t)(H - 1) * jslot));
    }
    return BAGEL_OK;
}

// Forward pass and loss; xi == null: pathwise function samples, else per-step posterior draws xi[H][B][M]
static int rollout_loss_impl(bagel_ctx *c, const char *who, const float *theta, const float *s0, const float *goals,
                             const float *xi, bool posterior, float *loss, float *loss_per_traj, float *states)
{
    if (!c) return BAGEL_EINVAL;
    c->err[0] = 0;
    if (!theta || !s0 || !goals || !loss || (posterior && !xi)) BAGEL_FAIL(c, BAGEL_EINVAL, "%s: null argument", who);
    if (posterior ? !c->post_prepared : !c->prepared)
        BAGEL_FAIL(c, BAGEL_ENOTPREPARED, "%s: %s", who, posterior ? "no posterior cache installed" : "no samples installed");
    c->cur_xi = posterior ? xi : nullptr;
    BAGEL_HIP(c, bagel_launch_pack_theta(c, theta));
    BAGEL_HIP(c, bagel_launch_init_state(c, s0, goals, states, false));
    const int rc = run_forward(c, false, false, false, theta, goals, states);
    if (rc != BAGEL_OK) return rc;
    BAGEL_HIP(c, bagel_launch_finish_loss(c, loss, loss_per_traj));
    return BAGEL_OK;
}

extern "C" int bagel_rollout_loss(bagel_ctx *c, const float *theta, const float *s0, const float *goals,
                                  float *loss, float *loss_per_traj, float *states)
{
    return rollout_loss_impl(c, "bagel_rollout_loss", theta, s0, goals, nullptr, false, loss, loss_per_traj, states);
}

extern "C" int bagel_posterior_rollout_loss(bagel_ctx *c, const float *theta, const float *s0, const float *goals,
                                            const float *xi, float *loss, float *loss_per_traj, float *states)
{
    return rollout_loss_impl(c, "bagel_posterior_rollout_loss", theta, s0, goals, xi, true, loss, loss_per_traj, states);
}

static int rollout_loss_grad_impl(bagel_ctx *c, const char *who, const float *theta, const float *s0,
                                  const float *goals, const float *xi, bool posterior, float *loss, float *grad_theta,
                                  float *loss_per_traj, float *states, float *grad_s0)
{
    if (!c) return BAGEL_EINVAL;
    c->err[0] = 0;
    if (!theta || !s0 || !goals || !loss || !grad_theta || (posterior && !xi))
        BAGEL_FAIL(c, BAGEL_EINVAL, "%s: null argument", who);
    if (posterior ? !c->post_prepared : !c->prepared)
        BAGEL_FAIL(c, BAGEL_ENOTPREPARED, "%s: %s", who, posterior ? "no posterior cache installed" : "no samples installed");
    c->cur_xi = posterior ? xi : nullptr;
    const int H = c->dm.H, K = c->T_tape;
    const bool ckpt = K < H;
    int rc;
    BAGEL_HIP(c, bagel_launch_pack_theta(c, theta));
    BAGEL_HIP(c, bagel_launch_init_state(c, s0, goals, states, true));
    // One forward pass with Jacobians.  Without checkpointing it also keeps the policy's activations.
    rc = run_forward(c, true, !ckpt, true, theta, goals, states);
    if (rc != BAGEL_OK) return rc;
    BAGEL_HIP(c, bagel_launch_finish_loss(c, loss, loss_per_traj));
    if (!ckpt) {
        BAGEL_HIP(c, bagel_launch_backward_sweep(c, 0, H, goals, grad_s0));
        BAGEL_HIP(c, bagel_launch_weight_grad(c, H, false, grad_theta));
        return BAGEL_OK;
    }
    // Checkpointed (Sec. IV-C): what is large, the activations and adjoints of the policy (about 4 KB
    // per trajectory and step with 256-wide layers), is held for one segment of K steps at a time and
    // rebuilt from the kept float32 states, all steps of the segment in one launch; what is small and
    // expensive to recompute, the state (d_s floats) and the Jacobian of the sample evaluation (M D
    // floats), is kept for the whole horizon.  Segments are swept from the last to the first.
    // Only the sweep is a chain from segment to segment (the adjoint of the state); the replay of a
    // segment needs the kept states alone and the weight gradient of a segment only that segment's
    // tapes.  The sweep occupies one workgroup per 32 trajectories for a whole segment, which leaves
    // compute units idle below 8192 trajectories, so the other two run beside it on a second stream
    // and a second set of tapes:  main: S(n-1) S(n-2) S(n-3) ...;  side: R(n-1) R(n-2) W(n-1) R(n-3) W(n-2) ...
    // S(k) waits for R(k); W(k) waits for S(k); R(k-1), which reuses the tapes of segment k+1, follows
    // W(k+1) in stream order.  The weight gradients are still added up in segment order, on one stream.
    const int n_seg = (H + K - 1) / K;
    const hipStream_t main_stream = c->stream;
    hipError_t e = hipSuccess;
    auto on_side = [&](int seg, bool replay) {
        const int t0 = seg * K, t1 = (t0 + K < H) ? t0 + K : H;
        use_tape_set(c, seg & 1);
        c->stream = c->side;
        hipError_t r = replay ? bagel_launch_policy_replay(c, t0, t1, theta, goals)
                              : bagel_launch_weight_grad(c, t1 - t0, seg != n_seg - 1, seg == 0 ? grad_theta : nullptr);
        c->stream = main_stream;
        if (r == hipSuccess && replay) r = hipEventRecord(c->ev_replay[seg & 1], c->side);
        return r;
    };
    e = hipEventRecord(c->ev_fork, main_stream);
    if (e == hipSuccess) e = hipStreamWaitEvent(c->side, c->ev_fork, 0);
    if (e == hipSuccess) e = on_side(n_seg - 1, true);
    for (int seg = n_seg - 1; seg >= 0 && e == hipSuccess; --seg) {
        const int t0 = seg * K, t1 = (t0 + K < H) ? t0 + K : H, set = seg & 1;
        e = hipStreamWaitEvent(main_stream, c->ev_replay[set], 0);
        use_tape_set(c, set);
        if (e == hipSuccess) e = bagel_launch_backward_sweep(c, t0, t1, goals, grad_s0);
        if (e == hipSuccess) e = hipEventRecord(c->ev_sweep[set], main_stream);
        if (e == hipSuccess && seg > 0) e = on_side(seg - 1, true);
        if (e == hipSuccess) e = hipStreamWaitEvent(c->side, c->ev_sweep[set], 0);
        if (e == hipSuccess) e = on_side(seg, false);
    }
    // the caller's stream continues after the last weight gradient
    if (e == hipSuccess) e = hipEventRecord(c->ev_join, c->side);
    if (e == hipSuccess) e = hipStreamWaitEvent(main_stream, c->ev_join, 0);
    use_tape_set(c, 0);
    if (e != hipSuccess) BAGEL_FAIL(c, BAGEL_EHIP, "%s: checkpointed backward pass failed: %s", who, hipGetErrorString(e));
    return BAGEL_OK;
}

extern "C" int bagel_rollout_loss_grad(bagel_ctx *c, const float *theta, const float *s0, const float *goals,
                                       float *loss, float *grad_theta, float *loss_per_traj, float *states,
                                       float *grad_s0)
{
    return rollout_loss_grad_impl(c, "bagel_rollout_loss_grad", theta, s0, goals, nullptr, false, loss, grad_theta,
                                  loss_per_traj, states, grad_s0);
}

extern "C" int bagel_posterior_rollout_loss_grad(bagel_ctx *c, const float *theta, const float *s0, const float *goals,
                                                 const float *xi, float *loss, float *grad_theta,
                                                 float *loss_per_traj, float *states, float *grad_s0)
{
    return rollout_loss_grad_impl(c, "bagel_posterior_rollout_loss_grad", theta, s0, goals, xi, true, loss, grad_theta,
                                  loss_per_traj, states, grad_s0);
}

// Exact posterior cache for the per-step sampler.  The first call allocates it.
extern "C" int bagel_prepare_posterior(bagel_ctx *c, const float *X, const float *y, const float *lengthscale,
                                       const float *signal_var, const float *noise_var)
{
    if (!c) return BAGEL_EINVAL;
    c->err[0] = 0;
    if (!X || !y || !lengthscale || !signal_var || !noise_var)
        BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_prepare_posterior: null argument");
    c->post_prepared = false;
    c->prepared = false;            // the scaled training inputs are rewritten below: installed samples belong to the old model
    if (!c->post_Kinv) {
        c->post_Np = (c->dm.N + 63) / 64 * 64;
        const size_t Np = (size_t)c->post_Np, B = (size_t)c->dm.B, M = (size_t)c->M;
        hipError_t e = dev_alloc(c, &c->post_alpha, M * Np);
        if (e == hipSuccess) e = dev_alloc(c, &c->post_Kinv, M * Np * Np);
        if (e == hipSuccess) e = dev_alloc(c, &c->post_Kx, M * Np * B);
        if (e == hipSuccess) e = dev_alloc(c, &c->post_sums, M * (Np / 64) * 2 * (1 + (size_t)c->D) * B);
        if (e != hipSuccess) {
            void *ptrs[] = {c->post_alpha, c->post_Kinv, c->post_Kx, c->post_sums};
            for (void *p : ptrs)
                if (p) (void)hipFree(p);
            c->post_alpha = c->post_Kinv = c->post_Kx = c->post_sums = nullptr;
            (void)hipGetLastError();
            BAGEL_FAIL(c, BAGEL_ENOMEM, "bagel_prepare_posterior: device allocation failed (%zu bytes for K_hat^-1)",
                       M * Np * Np * sizeof(double));
        }
    }
    // the scaled training inputs the kernel rows are computed from (the feature tables are left alone)
    BAGEL_HIP(c, bagel_launch_build_model(c, X, lengthscale, signal_var, nullptr, nullptr));
    const int rc = bagel_prepare_posterior_impl(c, X, y, lengthscale, signal_var, noise_var);
    if (rc != BAGEL_OK) return rc;
    c->post_prepared = true;
    return BAGEL_OK;
}

static const char *check_adam(int step, float lr, float beta1, float beta2, float eps)
{
    if (step < 1) return "step must be >= 1";
    if (!(lr > 0.0f) || !(eps > 0.0f)) return "lr and eps must be positive";
    if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f)) return "betas must lie in [0, 1)";
    return nullptr;
}

static hipError_t adam_update(bagel_ctx *c, float *theta, const float *grad, float *m, float *v, int step,
                              float lr, float beta1, float beta2, float eps)
{
    const double b1 = (double)beta1, b2 = (double)beta2;
    return bagel_launch_adam(c, theta, grad, m, v, c->P, (double)lr, b1, b2, (double)eps, 1.0 - pow(b1, (double)step),
                             1.0 - pow(b2, (double)step));
}

extern "C" int bagel_adam_step(bagel_ctx *c, float *theta, const float *grad, float *adam_m, float *adam_v,
                               int step, float lr, float beta1, float beta2, float eps)
{
    if (!c) return BAGEL_EINVAL;
    c->err[0] = 0;
    if (!theta || !grad || !adam_m || !adam_v) BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_adam_step: null argument");
    if (const char *msg = check_adam(step, lr, beta1, beta2, eps)) BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_adam_step: %s", msg);
    BAGEL_HIP(c, adam_update(c, theta, grad, adam_m, adam_v, step, lr, beta1, beta2, eps));
    return BAGEL_OK;
}

extern "C" int bagel_optimize(bagel_ctx *c, float *theta, float *adam_m, float *adam_v, const float *s0_sets,
                              const float *goal_sets, int n_sets, int n_iters, int first_step, float lr,
                              float beta1, float beta2, float eps, float *loss_history)
{
    if (!c) return BAGEL_EINVAL;
    c->err[0] = 0;
    if (!theta || !adam_m || !adam_v || !s0_sets || !goal_sets || !loss_history)
        BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_optimize: null argument");
    if (n_sets < 1 || n_iters < 0) BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_optimize: n_sets must be >= 1 and n_iters >= 0");
    if (const char *msg = check_adam(first_step, lr, beta1, beta2, eps)) BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_optimize: %s", msg);
    if (!c->prepared) BAGEL_FAIL(c, BAGEL_ENOTPREPARED, "bagel_optimize: no samples installed");
    const size_t s0_sz = (size_t)c->dm.B * c->dm.d_s, g_sz = (size_t)c->dm.H * c->dm.B * c->dm.d_g;
    for (int i = 0; i < n_iters; ++i) {
        const int set = i % n_sets;
        const int rc = bagel_rollout_loss_grad(c, theta, s0_sets + set * s0_sz, goal_sets + set * g_sz, loss_history + i,
                                               c->gtheta, nullptr, nullptr, nullptr);
        if (rc != BAGEL_OK) return rc;
        BAGEL_HIP(c, adam_update(c, theta, c->gtheta, adam_m, adam_v, first_step + i, lr, beta1, beta2, eps));
    }
    return BAGEL_OK;
}

extern "C" int bagel_hyper_lml_grad(bagel_ctx *c, const float *X, const float *y, const float *log_hyp, float *lml,
                                    float *grad)
{
    if (!c) return BAGEL_EINVAL;
    c->err[0] = 0;
    if (!X || !y || !log_hyp || !lml) BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_hyper_lml_grad: null argument");
    return bagel_hyper_impl(c, X, y, const_cast<float *>(log_hyp), lml, grad, nullptr, nullptr, 0, 1, 0.0, 0.0, 0.0, 0.0);
}

extern "C" int bagel_hyper_fit(bagel_ctx *c, const float *X, const float *y, float *log_hyp, float *adam_m,
                               float *adam_v, int n_iters, int first_step, float lr, float beta1, float beta2,
                               float eps, float *lml_history)
{
    if (!c) return BAGEL_EINVAL;
    c->err[0] = 0;
    if (!X || !y || !log_hyp || !adam_m || !adam_v || !lml_history)
        BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_hyper_fit: null argument");
    if (n_iters < 1) BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_hyper_fit: n_iters must be >= 1");
    if (const char *msg = check_adam(first_step, lr, beta1, beta2, eps)) BAGEL_FAIL(c, BAGEL_EINVAL, "bagel_hyper_fit: %s", msg);
    return bagel_hyper_impl(c, X, y, log_hyp, lml_history, nullptr, adam_m, adam_v, n_iters, first_step, (double)lr,
                            (double)beta1, (double)beta2, (double)eps);
}
