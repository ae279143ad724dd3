// Per-step posterior sampler: Algorithm 1 as printed draws the next state at every step from the
// predictive posterior of the GPs (eq. (9)), one independent GP per state increment (Sec. III-A):
//   f_m = mu_m(x) + sqrt(var_m(x)) xi_m,    xi ~ N(0, 1) supplied by the caller (reparameterised draw),
//   mu_m(x)  = k_m(x, X)^T alpha_m,                  alpha_m = K_hat_m^-1 y_m          (eq. (2), zero prior mean)
//   var_m(x) = alpha_m^2 - k_m(x, X)^T K_hat_m^-1 k_m(x, X)                             (eq. (3))
// with the exact K_hat^-1 from bagel_prepare_posterior (the paper speeds the variance up with Lanczos
// estimates of the same quantity; that approximation is not reproduced here).
//
// One step, all outputs m and all B trajectories at once:
//   1. posterior_rows_kernel: Kx[m][n][b] = k_m(x_b, X_n) in float64 (lane = trajectory, training inputs as
//      scalar operands, the same expanded-distance form and software exp2 as the pathwise step kernel);
//   2. posterior_gemm_kernel: Q = K_hat_m^-1 Kx_m, a float64 product [Np x Np] x [Np x B] per output and
//      the dominant cost (2 N^2 flop per trajectory, step and output).  Q is never written: the
//      workgroup that finishes a 64 x 64 tile of it multiplies the tile with the kernel rows and adds
//      up, over the tile's 64 training points, the sums the moments are made of,
//        sum_n a_n k_n, sum_n q_n k_n, sum_n a_n k_n Xs_nd, sum_n q_n k_n Xs_nd     (a = alpha_m, q = Q column),
//      one set per tile row and trajectory;
//   3. posterior_final_kernel adds the tile rows in order and finishes mu, var and their derivatives,
//        d mu / d x_d  = ln2 (sum_n a_n k_n Xs_nd - A_d x_d sum_n a_n k_n),
//        d var / d x_d = -2 ln2 (sum_n q_n k_n Xs_nd - A_d x_d sum_n q_n k_n),
//      then f and J = d mu + xi / (2 sqrt(var)) d var, written in the layout the end-of-step kernel reads.
// A variance below 1e-12 is held there and its derivative set to zero.
// Everything after that (state update, cost, tape, policy, backward sweep) is shared with the pathwise sampler.
#include "bagel_internal.h"
#include "dgemm_tile.h"

namespace {

constexpr double LN2 = 0.69314718055994530942;
constexpr double VAR_FLOOR = 1e-12;

struct bagel_post_sf2 {
    double v[8];                 // signal variance of every output
};

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

// Kx[m][n][b] for m = blockIdx.z, n in [32 blockIdx.y, +32), b = lane; rows n >= N (padding) are zero
template <int D>
__global__ __launch_bounds__(256) void posterior_rows_kernel(const double *__restrict__ Xs, const double *__restrict__ A,
                                                             const double *__restrict__ xbuf, double *__restrict__ Kx,
                                                             int B, int N, int Np, int Np_model)
{
    const int m = blockIdx.z;
    const double *__restrict__ Xs_m = Xs + (size_t)m * Np_model * (D + 1);
    const double *__restrict__ A_m = A + (size_t)m * D;
    double *__restrict__ Kx_m = Kx + (size_t)m * Np * B;
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
        if (live) Kx_m[(size_t)n * B + b] = k;
    }
}

// Tile (blockIdx.y, blockIdx.x) of Q_m = K_hat_m^-1 Kx_m for m = blockIdx.z, folded at once into the
// sums over the tile's 64 training points: sums[m][blockIdx.y][v][b], v = 0: sum a k, 1: sum q k,
// 2 + d: sum a k Xs_d, 2 + D + d: sum q k Xs_d.  Every sum is formed in a fixed order (a lane's eight
// rows, then the four lane groups, then the two waves that share the columns).
template <int D>
__global__ __launch_bounds__(256, (D <= 8 ? 4 : 2)) void posterior_gemm_kernel(const double *__restrict__ Kinv, const double *__restrict__ Kx,
                                                             const double *__restrict__ alpha,
                                                             const double *__restrict__ Xs, double *__restrict__ sums,
                                                             int B, int N, int Np, int Np_model)
{
    constexpr int NV = 2 * (1 + D);
    __shared__ bagel_gemm::tile_lds sh;
    __shared__ double red[2][2][NV][16];
    const int m = blockIdx.z;
    const int i0 = blockIdx.y * bagel_gemm::TM, j0 = blockIdx.x * bagel_gemm::TN;
    const double *__restrict__ Kx_m = Kx + (size_t)m * Np * B;
    const double *__restrict__ alpha_m = alpha + (size_t)m * Np;
    const double *__restrict__ Xs_m = Xs + (size_t)m * Np_model * (D + 1);
    bagel_gemm::d4v acc[2][2];
    bagel_gemm::tile_product(acc, sh, i0, j0, Np, B, Np, Kinv + (size_t)m * Np * Np, Np, 1, Kx_m, B, 1);
    // scaled inputs and alpha of the tile's 64 training points, into the LDS the product is done with
    // (zero on the padding rows); tile_product ended with a barrier
    constexpr int LW = D + 1;
    double *xl = reinterpret_cast<double *>(&sh);
    static_assert(64 * LW * sizeof(double) <= sizeof(bagel_gemm::tile_lds), "tile LDS too small for the staged rows");
    for (int idx = threadIdx.x; idx < 64 * LW; idx += 256) {
        const int row = idx / LW, col = idx - row * LW, gi = i0 + row;
        double val = 0.0;
        if (gi < N) val = col < D ? Xs_m[(size_t)gi * (D + 1) + col] : alpha_m[gi];
        xl[idx] = val;
    }
    __syncthreads();
    const bagel_gemm::lane_pos pos = bagel_gemm::lane_position();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = wave & 1;                        // which 32 columns of the tile
    double *__restrict__ out = sums + ((size_t)m * gridDim.y + blockIdx.y) * NV * B;
    // one of the lane's two columns at a time, to keep the sums within the register budget
#pragma unroll
    for (int y = 0; y < 2; ++y) {
        const int gj = j0 + pos.col0 + 16 * y;
        double kv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {                 // e = 4 x + r; padding rows of Kx are zero
            const int gi = i0 + pos.row0 + 16 * (e >> 2) + 4 * (e & 3);
            kv[e] = gj < B ? Kx_m[(size_t)gi * B + gj] : 0.0;
        }
        double s[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) s[v] = 0.0;
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const double *__restrict__ row = xl + (pos.row0 + 16 * x + 4 * r) * LW;
                const double k = kv[4 * x + r];
                const double ak = row[D] * k, qk = acc[x][y][r] * k;
                s[0] += ak;
                s[1] += qk;
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    s[2 + d] = fma(ak, row[d], s[2 + d]);
                    s[2 + D + d] = fma(qk, row[d], s[2 + D + d]);
                }
            }
        // the four lane groups of a wave hold different rows of the same columns
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            s[v] += __shfl_xor(s[v], 16);
            s[v] += __shfl_xor(s[v], 32);
        }
        // the waves of the lower half of the tile hand their sums to the waves of the upper half
        if ((wave >> 1) == 1 && lane < 16) {
#pragma unroll
            for (int v = 0; v < NV; ++v) red[half][y][v][lane] = s[v];
        }
        __syncthreads();
        if ((wave >> 1) == 0 && lane < 16 && gj < B) {
#pragma unroll
            for (int v = 0; v < NV; ++v) out[(size_t)v * B + gj] = s[v] + red[half][y][v][lane];
        }
    }
}

// Adds the tile rows in order and finishes the draw: thread = trajectory, blockIdx.y = component
// (0 -> f, 1 + d -> J[d]), blockIdx.z = output.  out[m][comp][b].
template <int D>
__global__ __launch_bounds__(256) void posterior_final_kernel(const double *__restrict__ sums, const double *__restrict__ A,
                                                              const double *__restrict__ xbuf,
                                                              const float *__restrict__ xi_t, bagel_post_sf2 sf2,
                                                              double *__restrict__ out, int B, int M, int ntile)
{
    constexpr int NV = 2 * (1 + D);
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    const int comp = blockIdx.y, d = comp - 1, m = blockIdx.z;
    const double *__restrict__ p = sums + (size_t)m * ntile * NV * B + b;
    double mu = 0.0, quad = 0.0, gmu = 0.0, gq = 0.0;
    for (int t = 0; t < ntile; ++t) {
        const double *__restrict__ pt = p + (size_t)t * NV * B;
        mu += pt[0];
        quad += pt[(size_t)B];
        if (comp > 0) {
            gmu += pt[(size_t)(2 + d) * B];
            gq += pt[(size_t)(2 + D + d) * B];
        }
    }
    double var = sf2.v[m] - quad;
    const bool floored = var < VAR_FLOOR;
    if (floored) var = VAR_FLOOR;
    const double sd = sqrt(var);
    const double z = (double)xi_t[(size_t)b * M + m];
    double *__restrict__ o = out + (size_t)m * (1 + D) * B;
    if (comp == 0) {
        o[b] = mu + sd * z;
    } else {
        const double ax = A[(size_t)m * D + d] * xbuf[(size_t)d * B + b];
        const double dmu = LN2 * (gmu - ax * mu);
        const double dvar = floored ? 0.0 : -2.0 * LN2 * (gq - ax * quad);
        o[(size_t)comp * B + b] = dmu + z * dvar / (2.0 * sd);
    }
}

template <int D>
hipError_t step_d(bagel_ctx *c, bool jac, const float *xi_t)
{
    const int B = c->dm.B, N = c->dm.N, Np = c->post_Np, M = c->M;
    const int ntile = Np / bagel_gemm::TM;
    bagel_post_sf2 sf2;
    for (int m = 0; m < 8; ++m) sf2.v[m] = c->post_sf2[m];
    hipLaunchKernelGGL((posterior_rows_kernel<D>), dim3((B + 255) / 256, (Np + 31) / 32, M), dim3(256), 0, c->stream,
                       c->Xs, c->A, c->xbuf, c->post_Kx, B, N, Np, c->Np);
    hipLaunchKernelGGL((posterior_gemm_kernel<D>), dim3((B + 63) / 64, ntile, M), dim3(256), 0, c->stream, c->post_Kinv,
                       c->post_Kx, c->post_alpha, c->Xs, c->post_sums, B, N, Np, c->Np);
    hipLaunchKernelGGL((posterior_final_kernel<D>), dim3((B + 255) / 256, jac ? 1 + D : 1, M), dim3(256), 0, c->stream,
                       c->post_sums, c->A, c->xbuf, xi_t, sf2, c->part, B, M, ntile);
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
