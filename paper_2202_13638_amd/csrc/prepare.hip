// Sample-set precompute: v_sm = (K_m + noise_m I)^-1 (y_m - Phi_m w_sm - eps_sm) for every
// function sample s and output m (Matheron update of a pathwise sample; K_hat as defined below
// eq. (3), kernel of eq. (4)).  Everything is float64 on the device: the condition number of
// K_hat is ~ signal/noise variance times N, far beyond float32.  Per output:
//   1. K_hat (padded to a multiple of 64 with an identity block) and Phi are built from the
//      float32 inputs;
//   2. recursively blocked Cholesky: 64x64 diagonal factorisation and panel solve inside ranges of
//      256 columns, the larger ranges updated by tiled float64 GEMMs as deep as half the range;
//   3. R = y 1^T - Phi W^T - Eps^T as one GEMM over the L features (R is [N][S]);
//   4. blocked forward and backward substitution on all S right-hand sides at once, again
//      GEMM-dominated;
//   5. v is rounded to float32 once, written to v_out[S][M][N] and packed for the step kernel.
// This is set-up work outside the timed rollouts; buffers are allocated here and freed on return.
#include <math.h>
#include <stdio.h>

#include "bagel_internal.h"
#include "dgemm_tile.h"

namespace {

constexpr int NB = 64;    // Cholesky / substitution block
using bagel_gemm::TM;
using bagel_gemm::TN;

// K_hat[i][j] for i, j < Np (row-major, leading dimension Np); identity on the padding
__global__ void build_khat_kernel(const float *__restrict__ X, const float *__restrict__ ell, float sf2, float sn2,
                                  double *__restrict__ K, int N, int Np, int D)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int i = blockIdx.y;
    if (j >= Np) return;
    double val;
    if (i < N && j < N) {
        double r = 0.0;
        for (int d = 0; d < D; ++d) {
            const double t = ((double)X[(size_t)i * D + d] - (double)X[(size_t)j * D + d]) / (double)ell[d];
            r += t * t;
        }
        val = (double)sf2 * exp(-0.5 * r);
        if (i == j) val += (double)sn2;
    } else {
        val = (i == j) ? 1.0 : 0.0;
    }
    K[(size_t)i * Np + j] = val;
}

// Phi[n][l] = sqrt(2 sf2 / L) cos(omega_l . X_n + phase_l); zero rows on the padding
__global__ void build_phi_kernel(const float *__restrict__ X, const float *__restrict__ omega,
                                 const float *__restrict__ phase, float sf2, double *__restrict__ Phi, int N,
                                 int Np, int L, int D)
{
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    const int n = blockIdx.y;
    if (l >= L) return;
    double val = 0.0;
    if (n < N) {
        double z = (double)phase[l];
        for (int d = 0; d < D; ++d) z += (double)omega[(size_t)l * D + d] * (double)X[(size_t)n * D + d];
        val = sqrt(2.0 * (double)sf2 / (double)L) * cos(z);
    }
    Phi[(size_t)n * L + l] = val;
}

// R[n][s] = y[n] - eps[s][n] (zero on the padding); eps is [S][M][N] at output m
__global__ void init_rhs_kernel(const float *__restrict__ y_m, const float *__restrict__ eps, double *__restrict__ R,
                                int N, int Np, int S, int M, int m)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    const int n = blockIdx.y;
    if (s >= S) return;
    double val = 0.0;
    if (n < N) val = (double)y_m[n] - (double)eps[((size_t)s * M + m) * N + n];
    R[(size_t)n * S + s] = val;
}

// Wd[s][l] = w[s][m][l]
__global__ void convert_w_kernel(const float *__restrict__ w, double *__restrict__ Wd, int S, int M, int L, int m)
{
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    const int s = blockIdx.y;
    if (l < L) Wd[(size_t)s * L + l] = (double)w[((size_t)s * M + m) * L + l];
}

// C[i][j] (ldc) += alpha * sum_k A(i,k) * B(k,j), A(i,k) = A[i*sai + k*sak], B(k,j) = B[k*sbk + j*sbj]
// (C = alpha * ... with overwrite).  lower_only: skip tiles entirely above the diagonal j = i + diag
// (used for the symmetric products).  The tile product itself is in dgemm_tile.h.
__global__ __launch_bounds__(256, 4) void dgemm_kernel(int Mr, int Nc, int Kd, double alpha,
                                                    const double *__restrict__ A, long sai, long sak,
                                                    const double *__restrict__ Bm, long sbk, long sbj,
                                                    double *__restrict__ Cm, long ldc, int lower_only, int diag, int overwrite)
{
    const int i0 = blockIdx.y * TM, j0 = blockIdx.x * TN;
    if (lower_only && j0 > i0 + diag + TM - 1) return;
    __shared__ bagel_gemm::tile_lds sh;
    bagel_gemm::d4v acc[2][2];
    bagel_gemm::tile_product(acc, sh, i0, j0, Mr, Nc, Kd, A, sai, sak, Bm, sbk, sbj);
    const bagel_gemm::lane_pos pos = bagel_gemm::lane_position();
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int gi = i0 + pos.row0 + 16 * x + 4 * r;
                const int gj = j0 + pos.col0 + 16 * y;
                if (gi < Mr && gj < Nc) {
                    double *dst = Cm + (long)gi * ldc + gj;
                    *dst = (overwrite ? 0.0 : *dst) + alpha * acc[x][y][r];
                }
            }
}

// The kernels below work on 64 x 64 blocks with one wave, lane = row or column of the block, the
// lane's vector in registers and the shared triangular block in LDS, read as broadcasts.  What bounds
// them is the latency between an LDS read and the FMA that uses it, so every step requests the
// triangular row it needs as one burst of reads one step ahead (scheduling barriers keep the burst
// together) and then runs independent FMAs on values that have already arrived.
constexpr int LDB = NB + 2;      // LDS row stride: rows stay 16-byte aligned for two-element reads

// A 64 x 64 block of a row-major matrix <-> LDS, by one wave: lane = column, so every global access is
// one contiguous row; all 64 loads are requested before the first one is used.
template <bool TRANSPOSE>
__device__ __forceinline__ void block_to_lds(const double *__restrict__ src, size_t ld, double (*dst)[LDB])
{
    const int r = threadIdx.x;
    double t[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) t[i] = src[(size_t)i * ld + r];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        if (TRANSPOSE) dst[r][i] = t[i];
        else dst[i][r] = t[i];
    }
}

__device__ __forceinline__ void lds_to_block(double (*src)[LDB], double *__restrict__ dst, size_t ld)
{
    const int r = threadIdx.x;
#pragma unroll
    for (int i = 0; i < NB; ++i) dst[(size_t)i * ld + r] = src[i][r];
}

constexpr int CH = 16;           // entries of a triangular row requested per burst

// entries [16 q, 16 q + 16) of a row of the shared block, as one burst of broadcast reads
__device__ __forceinline__ void read_chunk(const double *row, int q, double (&dst)[CH])
{
#pragma unroll
    for (int e = 0; e < CH; ++e) dst[e] = row[q * CH + e];
}

// x <- L^-1 x for the lane's vector x, L lower triangular, given as its transpose Lt[i][c] = L[c][i]
// and the reciprocals of its diagonal: column by column, x[c] -= x[i] L[c][i] for c > i.
// The lane's vector takes half of the directly addressable registers, so the rows of Lt come in
// chunks of 16 entries, the next chunk in flight while the FMAs of the current one issue.
// One template instance per (row I, chunk Q): every register index is a compile-time constant.
template <int I, int Q, int IDX>
__device__ __forceinline__ void lower_item(double (&x)[NB], double (*Lt)[LDB], const double *rinv,
                                           double (&buf)[2][CH], double rc)
{
    constexpr int NQ = NB / CH;
    if constexpr (Q == (I + 1) / CH) x[I] *= rc;                  // first chunk of the row: x[I] is final
    constexpr bool same_row = Q + 1 < NQ;
    constexpr bool next_row = !same_row && (I + 2) / CH < NQ;     // row I + 1 has entries right of its diagonal
    double rn = rc;
    if constexpr (same_row) {
        read_chunk(Lt[I], Q + 1, buf[(IDX + 1) & 1]);
    } else {
        rn = rinv[I + 1];
        if constexpr (next_row) read_chunk(Lt[I + 1], (I + 2) / CH, buf[(IDX + 1) & 1]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int e = 0; e < CH; ++e) {
        const int c = Q * CH + e;
        if (c > I) x[c] = fma(-x[I], buf[IDX & 1][e], x[c]);
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (same_row) lower_item<I, Q + 1, IDX + 1>(x, Lt, rinv, buf, rc);
    else if constexpr (next_row) lower_item<I + 1, (I + 2) / CH, IDX + 1>(x, Lt, rinv, buf, rn);
    else x[I + 1] *= rn;                                         // the last row has nothing right of its diagonal
}

__device__ __forceinline__ void solve_lower(double (&x)[NB], double (*Lt)[LDB], const double *rinv)
{
    double buf[2][CH];
    read_chunk(Lt[0], 0, buf[0]);
    lower_item<0, 0, 0>(x, Lt, rinv, buf, rinv[0]);
}

// x <- L^-T x, L given by rows: from the last entry up, x[c] -= x[i] L[i][c] for c < i.
template <int I, int Q, int IDX>
__device__ __forceinline__ void upper_item(double (&x)[NB], double (*Ls)[LDB], const double *rinv,
                                           double (&buf)[2][CH], double rc)
{
    if constexpr (Q == 0) x[I] *= rc;
    constexpr bool same_row = Q + 1 <= (I - 1) / CH;
    constexpr bool next_row = !same_row && I - 1 >= 1;
    double rn = rc;
    if constexpr (same_row) {
        read_chunk(Ls[I], Q + 1, buf[(IDX + 1) & 1]);
    } else {
        rn = rinv[I - 1];
        if constexpr (next_row) read_chunk(Ls[I - 1], 0, buf[(IDX + 1) & 1]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int e = 0; e < CH; ++e) {
        const int c = Q * CH + e;
        if (c < I) x[c] = fma(-x[I], buf[IDX & 1][e], x[c]);
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (same_row) upper_item<I, Q + 1, IDX + 1>(x, Ls, rinv, buf, rc);
    else if constexpr (next_row) upper_item<I - 1, 0, IDX + 1>(x, Ls, rinv, buf, rn);
    else x[0] *= rn;
}

__device__ __forceinline__ void solve_lower_transposed(double (&x)[NB], double (*Ls)[LDB], const double *rinv)
{
    double buf[2][CH];
    read_chunk(Ls[NB - 1], 0, buf[0]);
    upper_item<NB - 1, 0, 0>(x, Ls, rinv, buf, rinv[NB - 1]);
}

// Step J of the factorisation of a diagonal block (see potrf_diag_kernel)
template <int J>
__device__ __forceinline__ void potrf_step(double (&a)[NB], double (*col)[NB], int r, int *__restrict__ flag,
                                           int flag_value)
{
    constexpr int NQ = NB / CH;
    const double d = __shfl(a[J], J);
    if (!(d > 0.0) && r == 0) atomicCAS(flag, 0, flag_value + J);
    // keep going with a harmless pivot so that the result stays finite
    const double piv = (d > 0.0) ? sqrt(d) : 1.0;
    const double l = (r == J) ? piv : a[J] / piv;
    a[J] = l;
    if constexpr (J + 1 < NB) {
        col[J & 1][r] = l;
        __syncthreads();
        // the column comes back in chunks of 16, the next chunk in flight under the FMAs of this one
        double buf[2][CH];
        constexpr int Q0 = (J + 1) / CH;
        read_chunk(col[J & 1], Q0, buf[Q0 & 1]);
#pragma unroll
        for (int q = Q0; q < NQ; ++q) {
            if (q + 1 < NQ) read_chunk(col[J & 1], q + 1, buf[(q + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int e = 0; e < CH; ++e) {
                const int c = q * CH + e;
                if (c > J) a[c] = fma(-l, buf[q & 1][e], a[c]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        potrf_step<J + 1>(a, col, r, flag, flag_value);
    }
}

// Factor the NB x NB diagonal block at (k,k) in place (lower).  Lane = row, the row lives in
// registers; right-looking: at step j the pivot comes from lane j, every lane scales its entry of
// column j, the column is broadcast through LDS and each lane updates the rest of its row with
// independent FMAs.  Entries above the diagonal are kept at zero, so no lane needs a predicate.
// Sets *flag = 1 + global row index on a pivot that is not positive.
__global__ __launch_bounds__(NB) void potrf_diag_kernel(double *__restrict__ K, int Np, int k, int flag_base,
                                                        int *__restrict__ flag)
{
    __shared__ __align__(16) double Ls[NB][LDB];
    __shared__ __align__(16) double col[2][NB];
    const int r = threadIdx.x;
    block_to_lds<false>(K + (size_t)k * Np + k, Np, Ls);
    __syncthreads();
    double a[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) a[c] = (c <= r) ? Ls[r][c] : 0.0;
    potrf_step<0>(a, col, r, flag, 1 + flag_base + k);
    __syncthreads();
#pragma unroll
    for (int c = 0; c < NB; ++c) Ls[r][c] = a[c];
    __syncthreads();
    lds_to_block(Ls, K + (size_t)k * Np + k, Np);
}

// Diagonal block L_kk into LDS (by rows, or transposed), with the reciprocals of its diagonal beside it
template <bool TRANSPOSE>
__device__ __forceinline__ void load_diag_block(const double *__restrict__ K, int Np, int k, double (*Ls)[LDB],
                                                double *rinv)
{
    block_to_lds<TRANSPOSE>(K + (size_t)k * Np + k, Np, Ls);
    __syncthreads();
    rinv[threadIdx.x] = 1.0 / Ls[threadIdx.x][threadIdx.x];
    __syncthreads();
}

// Panel solve: rows i >= k+NB of columns k..k+NB-1:  P <- P * L_kk^-T, which is a forward substitution
// with L_kk on every row of P.  One wave per 64 rows, lane = row; the rows go through LDS so that
// global accesses are coalesced.
__global__ __launch_bounds__(NB) void trsm_panel_kernel(double *__restrict__ K, int Np, int k)
{
    __shared__ __align__(16) double Lt[NB][LDB];
    __shared__ __align__(16) double Ps[NB][LDB];
    __shared__ double rinv[NB];
    load_diag_block<true>(K, Np, k, Lt, rinv);
    const int r = threadIdx.x;
    const int i0 = k + NB + blockIdx.x * NB;            // Np is a multiple of NB: the block of rows is whole
    block_to_lds<false>(K + (size_t)i0 * Np + k, Np, Ps);
    __syncthreads();
    double x[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) x[j] = Ps[r][j];
    solve_lower(x, Lt, rinv);
#pragma unroll
    for (int j = 0; j < NB; ++j) Ps[r][j] = x[j];
    __syncthreads();
    lds_to_block(Ps, K + (size_t)i0 * Np + k, Np);
}

// Forward substitution on block k for all right-hand sides: Z_k = L_kk^-1 R_k.  Lane = column s.
__global__ __launch_bounds__(NB) void trsv_fwd_kernel(const double *__restrict__ K, int Np, int k,
                                                      double *__restrict__ R, int S)
{
    __shared__ __align__(16) double Lt[NB][LDB];
    __shared__ double rinv[NB];
    load_diag_block<true>(K, Np, k, Lt, rinv);
    const int s = blockIdx.x * NB + threadIdx.x;
    if (s >= S) return;
    double z[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) z[i] = R[(size_t)(k + i) * S + s];
    solve_lower(z, Lt, rinv);
#pragma unroll
    for (int i = 0; i < NB; ++i) R[(size_t)(k + i) * S + s] = z[i];
}

// Backward substitution on block k: V_k = L_kk^-T Z_k.
__global__ __launch_bounds__(NB) void trsv_bwd_kernel(const double *__restrict__ K, int Np, int k,
                                                      double *__restrict__ R, int S)
{
    __shared__ __align__(16) double Ls[NB][LDB];
    __shared__ double rinv[NB];
    load_diag_block<false>(K, Np, k, Ls, rinv);
    const int s = blockIdx.x * NB + threadIdx.x;
    if (s >= S) return;
    double z[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) z[i] = R[(size_t)(k + i) * S + s];
    solve_lower_transposed(z, Ls, rinv);
#pragma unroll
    for (int i = 0; i < NB; ++i) R[(size_t)(k + i) * S + s] = z[i];
}

// V[n][s] (float64) -> v_out[s][m][n] (float32) and the packed stream v4[m][n4][s]
__global__ void emit_v_kernel(const double *__restrict__ V, float *__restrict__ v_out, float4 *__restrict__ v4,
                              int N, int Npk, int S, int M, int m)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    const int n4 = blockIdx.y;
    if (s >= S) return;
    float t[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int n = n4 * 4 + j;
        t[j] = n < N ? (float)V[(size_t)n * S + s] : 0.0f;
        if (v_out && n < N) v_out[((size_t)s * M + m) * N + n] = t[j];
    }
    v4[((size_t)m * (Npk / 4) + n4) * S + s] = make_float4(t[0], t[1], t[2], t[3]);
}

void gemm(hipStream_t st, int Mr, int Nc, int Kd, double alpha, const double *A, long sai, long sak,
          const double *Bm, long sbk, long sbj, double *Cm, long ldc, bool lower_only, bool overwrite = false,
          int diag = 0)
{
    if (Mr <= 0 || Nc <= 0 || Kd <= 0) return;
    dim3 grid((Nc + TN - 1) / TN, (Mr + TM - 1) / TM);
    hipLaunchKernelGGL(dgemm_kernel, grid, dim3(256), 0, st, Mr, Nc, Kd, alpha, A, sai, sak, Bm, sbk, sbj, Cm, ldc,
                       lower_only ? 1 : 0, diag, overwrite ? 1 : 0);
}

// In-place blocked Cholesky of K [Np][Np] (lower; Np a multiple of NB), then K_hat^-1 applied to the S
// right-hand sides R [Np][S] in place.  A pivot that is not positive is reported through *flag.
// Recursive blocking: a range of columns (or of unknowns) is split in halves, the first half is done,
// one product as deep as that half updates the second half, then the second half is done; ranges of
// at most OB columns advance in steps of NB with the one-wave block kernels.  A product only NB deep
// reads and writes every element it updates for NB multiply-adds on it, which is bound by memory
// traffic; the deep products of the upper levels, which carry most of the work, are bound by the
// matrix pipe.  (Flat blocking with 256-deep updates: 283 ms per hyper-parameter iteration at
// N = 8192; 512 deep: 270 ms; 1024 deep: 278 ms.)
constexpr int OB = 256;

struct solver {
    hipStream_t st;
    double *K;
    int Np;
    double *R;
    int S;
    int flag_base;
    int *flag;

    static int half(int n) { return (n / NB + 1) / 2 * NB; }       // first part of a split, a multiple of NB

    // columns [k, k + w) of the factor, for all rows down to Np
    void panel(int k, int w)
    {
        if (w > OB) {
            const int h = half(w);
            panel(k, h);
            // K[i][j] -= sum_c P[i][c] P[j][c] for i >= j in the rest of the range, P = columns [k, k + h)
            const double *Pn = K + (size_t)(k + h) * Np + k;
            gemm(st, Np - k - h, w - h, h, -1.0, Pn, Np, 1, Pn, 1, Np, K + (size_t)(k + h) * Np + (k + h), Np, true);
            panel(k + h, w - h);
            return;
        }
        for (int kk = k; kk < k + w; kk += NB) {
            hipLaunchKernelGGL(potrf_diag_kernel, dim3(1), dim3(NB), 0, st, K, Np, kk, flag_base, flag);
            const int below = Np - kk - NB;
            if (below <= 0) continue;
            hipLaunchKernelGGL(trsm_panel_kernel, dim3(below / NB), dim3(NB), 0, st, K, Np, kk);
            const int cols = k + w - kk - NB;           // columns of the range still to be factored
            const double *Pn = K + (size_t)(kk + NB) * Np + kk;
            if (cols > 0)
                gemm(st, below, cols, NB, -1.0, Pn, Np, 1, Pn, 1, Np, K + (size_t)(kk + NB) * Np + (kk + NB), Np, true);
        }
    }

    // forward substitution L Z = R on the unknowns [k, k + n); the rows below are updated by the caller
    void forward(int k, int n)
    {
        if (n > OB) {
            const int h = half(n);
            forward(k, h);
            gemm(st, n - h, S, h, -1.0, K + (size_t)(k + h) * Np + k, Np, 1, R + (size_t)k * S, S, 1,
                 R + (size_t)(k + h) * S, S, false);
            forward(k + h, n - h);
            return;
        }
        for (int kk = k; kk < k + n; kk += NB) {
            hipLaunchKernelGGL(trsv_fwd_kernel, dim3((S + NB - 1) / NB), dim3(NB), 0, st, K, Np, kk, R, S);
            const int rows = k + n - kk - NB;
            if (rows > 0)
                gemm(st, rows, S, NB, -1.0, K + (size_t)(kk + NB) * Np + kk, Np, 1, R + (size_t)kk * S, S, 1,
                     R + (size_t)(kk + NB) * S, S, false);
        }
    }

    // The same with R = identity (S = Np columns): Z = L^-1 is lower triangular, so while the unknowns
    // [k, k + n) are worked on only the columns below k + n hold anything; the products and block
    // solves stop there, which leaves N^3/4 of the N^3/2 multiply-adds of the general case.
    void forward_identity(int k, int n)
    {
        if (n > OB) {
            const int h = half(n);
            forward_identity(k, h);
            gemm(st, n - h, k + h, h, -1.0, K + (size_t)(k + h) * Np + k, Np, 1, R + (size_t)k * S, S, 1,
                 R + (size_t)(k + h) * S, S, false);
            forward_identity(k + h, n - h);
            return;
        }
        for (int kk = k; kk < k + n; kk += NB) {
            hipLaunchKernelGGL(trsv_fwd_kernel, dim3((kk + NB) / NB), dim3(NB), 0, st, K, Np, kk, R, S);
            const int rows = k + n - kk - NB;
            if (rows > 0)
                gemm(st, rows, kk + NB, NB, -1.0, K + (size_t)(kk + NB) * Np + kk, Np, 1, R + (size_t)kk * S, S, 1,
                     R + (size_t)(kk + NB) * S, S, false);
        }
    }

    // backward substitution L^T V = Z on the unknowns [k, k + n)
    void backward(int k, int n)
    {
        if (n > OB) {
            const int h = half(n);
            backward(k + h, n - h);
            // R[k : k+h] -= L[k+h : k+n, k : k+h]^T V[k+h : k+n] : A(i, c) = K[(k+h+c)*Np + k + i]
            gemm(st, h, S, n - h, -1.0, K + (size_t)(k + h) * Np + k, 1, Np, R + (size_t)(k + h) * S, S, 1,
                 R + (size_t)k * S, S, false);
            backward(k, h);
            return;
        }
        for (int kk = k + n - NB; kk >= k; kk -= NB) {
            hipLaunchKernelGGL(trsv_bwd_kernel, dim3((S + NB - 1) / NB), dim3(NB), 0, st, K, Np, kk, R, S);
            if (kk > k)   // R[k:kk] -= L[kk:kk+NB, k:kk]^T V_kk : A(i, c) = K[(kk+c)*Np + k + i]
                gemm(st, kk - k, S, NB, -1.0, K + (size_t)kk * Np + k, 1, Np, R + (size_t)kk * S, S, 1,
                     R + (size_t)k * S, S, false);
        }
    }
};

void factor_and_solve(hipStream_t st, double *K, int Np, double *R, int S, int flag_base, int *flag)
{
    solver s{st, K, Np, R, S, flag_base, flag};
    s.panel(0, Np);
    s.forward(0, Np);
    s.backward(0, Np);
}

// Z = identity [Np][Np]; yd[n] = y[n] in float64 (zero on the padding)
__global__ void inverse_init_kernel(const float *__restrict__ y_m, double *__restrict__ Z, double *__restrict__ yd, int N,
                                    int Np)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int n = blockIdx.y;
    if (j >= Np) return;
    Z[(size_t)n * Np + j] = (j == n) ? 1.0 : 0.0;
    if (n == 0) yd[j] = (j < N) ? (double)y_m[j] : 0.0;
}

// A[j][i] = A[i][j] for j > i, 32 x 32 blocks through LDS so that reads and writes are both row segments
__global__ __launch_bounds__(256) void mirror_lower_kernel(double *__restrict__ A, int Np)
{
    __shared__ double t[32][33];
    const int bi = blockIdx.y, bj = blockIdx.x;      // source block (rows bi, columns bj), bj <= bi
    if (bj > bi) return;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int r = ty; r < 32; r += 8) t[r][tx] = A[(size_t)(32 * bi + r) * Np + 32 * bj + tx];
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int row = 32 * bj + r, col = 32 * bi + tx;          // destination (row, col) = source (col, row)
        if (col > row) A[(size_t)row * Np + col] = t[tx][r];
    }
}

// out[i] = sum_k A[i][k] y[k] for a square row-major matrix: one wave per row, the lanes walk the row
// together (contiguous reads), their sums are added by a fixed butterfly.
__global__ __launch_bounds__(256) void matrix_times_vector_kernel(const double *__restrict__ A, const double *__restrict__ y,
                                                                  double *__restrict__ out, int Np)
{
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= Np) return;
    const double *row = A + (size_t)i * Np;
    double s = 0.0;
    for (int k = lane; k < Np; k += 64) s += row[k] * y[k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (lane == 0) out[i] = s;
}

// K_hat^-1 and alpha = K_hat^-1 y from the factor L in K (eq. (2), (3), (5), (6) all need both):
// Z = L^-1 by structured forward substitution on the identity, K_hat^-1 = Z^T Z on and below the
// diagonal in row panels (entry (i, j) only sums over k >= max(i, j), so a panel that starts at row
// i0 contracts over Np - i0 rows of Z), mirrored into the upper triangle; alpha = K_hat^-1 y as a
// matrix-vector product.  N^3/4 + N^3/6 multiply-adds after the N^3/6 of the factorisation, against N^3
// for substitution both ways on N right-hand sides.  Z [Np][Np] and yd [Np] are work space; Kinv and
// alpha the results.
constexpr int INV_PANEL = 512;

void inverse_from_factor(hipStream_t st, double *K, int Np, double *Z, const float *y_m, int N, double *yd, double *Kinv,
                         double *alpha, int flag_base, int *flag)
{
    hipLaunchKernelGGL(inverse_init_kernel, dim3((Np + 255) / 256, Np), dim3(256), 0, st, y_m, Z, yd, N, Np);
    solver s{st, K, Np, Z, Np, flag_base, flag};
    s.panel(0, Np);
    s.forward_identity(0, Np);
    for (int i0 = 0; i0 < Np; i0 += INV_PANEL) {
        const int hb = Np - i0 < INV_PANEL ? Np - i0 : INV_PANEL;
        // Kinv[i0 + i][j] = sum_k Z[i0 + k][i0 + i] Z[i0 + k][j], j <= i0 + i
        gemm(st, hb, i0 + hb, Np - i0, 1.0, Z + (size_t)i0 * Np + i0, 1, Np, Z + (size_t)i0 * Np, Np, 1,
             Kinv + (size_t)i0 * Np, Np, true, true, i0);
    }
    hipLaunchKernelGGL(mirror_lower_kernel, dim3(Np / 32, Np / 32), dim3(256), 0, st, Kinv, Np);
    hipLaunchKernelGGL(matrix_times_vector_kernel, dim3((Np + 3) / 4), dim3(256), 0, st, Kinv, yd, alpha, Np);
}

// ---- hyper-parameter learning: log marginal likelihood and its gradient (eq. (5), (6)) ----------
// K_hat for hyper-parameters given as logarithms on the device: lh = (log l_1 .. log l_D, log alpha^2,
// log sigma_n^2); identity on the padding
__global__ void build_khat_log_kernel(const float *__restrict__ X, const float *__restrict__ lh, double *__restrict__ K,
                                      int N, int Np, int D)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int i = blockIdx.y;
    if (j >= Np) return;
    double inv_l[BAGEL_MAX_D];                       // 1 / l_d, once per thread
    for (int d = 0; d < D; ++d) inv_l[d] = exp(-(double)lh[d]);
    const double sf2 = exp((double)lh[D]), sn2 = exp((double)lh[D + 1]);
    double val;
    if (i < N && j < N) {
        double r = 0.0;
        for (int d = 0; d < D; ++d) {
            const double t = ((double)X[(size_t)i * D + d] - (double)X[(size_t)j * D + d]) * inv_l[d];
            r += t * t;
        }
        val = sf2 * exp(-0.5 * r);
        if (i == j) val += sn2;
    } else {
        val = (i == j) ? 1.0 : 0.0;
    }
    K[(size_t)i * Np + j] = val;
}

// fixed-order sum of one value per thread over a workgroup of 256 (result valid in thread 0)
__device__ __forceinline__ double block_sum_256(double v, double *sh)
{
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    return sh[0];
}

// lml = -1/2 y^T a - sum_i log L_ii - N/2 log(2 pi); L = factor in K (diagonal), a = alpha
__global__ __launch_bounds__(256) void hyper_lml_kernel(const double *__restrict__ Lf, const double *__restrict__ alpha,
                                                        const float *__restrict__ y_m, int N, int Np,
                                                        float *__restrict__ lml_out)
{
    __shared__ double sh[256];
    double ld = 0.0, quad = 0.0;
    for (int i = threadIdx.x; i < Np; i += 256) ld += log(Lf[(size_t)i * Np + i]);
    for (int n = threadIdx.x; n < N; n += 256) quad += (double)y_m[n] * alpha[n];
    const double ld_tot = block_sum_256(ld, sh);
    __syncthreads();
    const double q_tot = block_sum_256(quad, sh);
    if (threadIdx.x == 0) lml_out[0] = (float)(-0.5 * q_tot - ld_tot - 0.5 * (double)N * 1.8378770664093453);
}

// row i of sum_ij (a_i a_j - Kinv_ij) dK_hat_ij / dphi_c for c = 0 .. D+1 -> partial[i][D+2]
// (eq. (6) with dK/dlog l_d = K (x_d - x'_d)^2 / l_d^2, dK/dlog alpha^2 = K, dK_hat/dlog sigma_n^2 = sigma_n^2 I).
// One workgroup per row; thread t takes columns t, t + 256, ...; the D + 2 sums are added over the
// lanes of a wave by a fixed butterfly, then over the four waves in order.  All loops over d have the
// compile-time bound BAGEL_MAX_D so that the per-thread arrays stay in registers.
__global__ __launch_bounds__(256) void hyper_grad_rows_kernel(const float *__restrict__ X, const float *__restrict__ lh,
                                                              const double *__restrict__ Kinv,
                                                              const double *__restrict__ alpha,
                                                              double *__restrict__ partial, int N, int Np, int D)
{
    __shared__ double sh[4][BAGEL_MAX_D + 2];
    const int i = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    double acc[BAGEL_MAX_D + 2], inv_l[BAGEL_MAX_D], xi[BAGEL_MAX_D];
#pragma unroll
    for (int c = 0; c < BAGEL_MAX_D + 2; ++c) acc[c] = 0.0;
#pragma unroll
    for (int d = 0; d < BAGEL_MAX_D; ++d) {          // 1 / l_d and the row's own input, once per thread
        inv_l[d] = d < D ? exp(-(double)lh[d]) : 0.0;
        xi[d] = d < D ? (double)X[(size_t)i * D + d] : 0.0;
    }
    const double sf2 = exp((double)lh[D]), sn2 = exp((double)lh[D + 1]);
    const double ai = alpha[i];
    for (int j = threadIdx.x; j < N; j += 256) {
        const double w = ai * alpha[j] - Kinv[(size_t)i * Np + j];
        double r = 0.0, t2[BAGEL_MAX_D];
#pragma unroll
        for (int d = 0; d < BAGEL_MAX_D; ++d) {
            if (d < D) {
                const double t = (xi[d] - (double)X[(size_t)j * D + d]) * inv_l[d];
                t2[d] = t * t;
                r += t2[d];
            }
        }
        const double wk = w * sf2 * exp(-0.5 * r);
#pragma unroll
        for (int d = 0; d < BAGEL_MAX_D; ++d)
            if (d < D) acc[d] += wk * t2[d];
        acc[BAGEL_MAX_D] += wk;
        if (j == i) acc[BAGEL_MAX_D + 1] += w * sn2;
    }
#pragma unroll
    for (int c = 0; c < BAGEL_MAX_D + 2; ++c) {
        if (c < D || c >= BAGEL_MAX_D) {
            double v = acc[c];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
            if (lane == 0) sh[wave][c] = v;
        }
    }
    __syncthreads();
    // thread c < D writes the length-scale sums, threads BAGEL_MAX_D and BAGEL_MAX_D + 1 the other two
    const int c = threadIdx.x;
    if (c < D || c == BAGEL_MAX_D || c == BAGEL_MAX_D + 1) {
        const double tot = ((sh[0][c] + sh[1][c]) + sh[2][c]) + sh[3][c];
        partial[(size_t)i * (D + 2) + (c < D ? c : D + (c - BAGEL_MAX_D))] = tot;
    }
}

// grad[c] = 1/2 sum_i partial[i][c]; neg_scaled[c] = -grad[c] / N for the Adam update.  One workgroup
// per hyper-parameter c: thread t adds rows t, t + 256, ... in order, then a fixed tree over the threads.
__global__ __launch_bounds__(256) void hyper_grad_final_kernel(const double *__restrict__ partial, int N, int D,
                                                               float *__restrict__ grad,
                                                               float *__restrict__ neg_scaled)
{
    __shared__ double sh[256];
    const int c = blockIdx.x;
    double s = 0.0;
    for (int i = threadIdx.x; i < N; i += 256) s += partial[(size_t)i * (D + 2) + c];
    s = 0.5 * block_sum_256(s, sh);
    if (threadIdx.x == 0) {
        if (grad) grad[c] = (float)s;
        if (neg_scaled) neg_scaled[c] = (float)(-s / (double)N);
    }
}

// The GP outputs are independent, and the work on one of them is a chain of small dependent kernels
// (diagonal blocks, panel solves) between its deep products: on its own it leaves the chip idle a third
// of the time.  So up to three outputs are worked on side by side, each on a stream of its own with
// buffers of its own; what one leaves idle the deep products of another fill.  The side streams start
// after everything already enqueued on the context's stream and the context's stream continues after
// them; all have the default priority.  (Four or six side by side were measured as well: 142 and 127 ms
// per hyper-parameter iteration at N = 8192 against 127 ms with three.)
struct side_lanes {
    static constexpr int MAXL = 3;
    int n = 0;
    hipStream_t st[MAXL] = {};
    hipEvent_t done[MAXL] = {};
    hipEvent_t start = nullptr;

    hipError_t open(int want)
    {
        if (want > MAXL) want = MAXL;
        if (want < 1) want = 1;
        hipError_t e = hipEventCreateWithFlags(&start, hipEventDisableTiming);
        for (int l = 0; l < want && e == hipSuccess; ++l) {
            e = hipStreamCreateWithFlags(&st[l], hipStreamNonBlocking);
            if (e == hipSuccess) e = hipEventCreateWithFlags(&done[l], hipEventDisableTiming);
            if (e == hipSuccess) n = l + 1;
        }
        return e;
    }
    hipError_t fork(hipStream_t main)
    {
        hipError_t e = hipEventRecord(start, main);
        for (int l = 0; l < n && e == hipSuccess; ++l) e = hipStreamWaitEvent(st[l], start, 0);
        return e;
    }
    hipError_t join(hipStream_t main)
    {
        hipError_t e = hipSuccess;
        for (int l = 0; l < n && e == hipSuccess; ++l) {
            e = hipEventRecord(done[l], st[l]);
            if (e == hipSuccess) e = hipStreamWaitEvent(main, done[l], 0);
        }
        return e;
    }
    void sync()
    {
        for (int l = 0; l < n; ++l) (void)hipStreamSynchronize(st[l]);
    }
    void close()
    {
        for (int l = 0; l < MAXL; ++l) {
            if (st[l]) { (void)hipStreamSynchronize(st[l]); (void)hipStreamDestroy(st[l]); }
            if (done[l]) (void)hipEventDestroy(done[l]);
        }
        if (start) (void)hipEventDestroy(start);
    }
};

// What the set-up calls need beyond the context's own buffers: the side streams and one device
// allocation that their float64 work space is carved from.  Both are made by the first set-up call,
// grown when a later call needs more, kept for the next call (a caller's own loop over
// bagel_hyper_lml_grad, or a redraw of the samples with bagel_prepare_samples every few policy
// updates, allocates nothing after its first pass) and released by bagel_destroy.
struct setup_scratch {
    side_lanes lanes;
    bool lanes_open = false;
    char *arena = nullptr;
    size_t arena_bytes = 0;
};

constexpr size_t ARENA_ALIGN = 256;
size_t arena_round(size_t bytes) { return (bytes + ARENA_ALIGN - 1) / ARENA_ALIGN * ARENA_ALIGN; }

// The context's set-up scratch with its side streams open (at most `want` of them) and at least
// shared_bytes + n * lane_bytes of device memory, n = number of outputs worked on side by side: as many
// as there are streams, fewer if the memory for that many cannot be had (one must fit).  The stream is
// idle when the arena is replaced: every set-up call ends with a synchronisation.
hipError_t setup_reserve(bagel_ctx *c, int want, size_t lane_bytes, size_t shared_bytes, setup_scratch **out, int *n_side)
{
    setup_scratch *sc = static_cast<setup_scratch *>(c->setup);
    if (!sc) {
        sc = new (std::nothrow) setup_scratch();
        if (!sc) return hipErrorOutOfMemory;
        c->setup = sc;
    }
    if (!sc->lanes_open) {
        const hipError_t e = sc->lanes.open(want);
        if (e != hipSuccess) {
            sc->lanes.close();
            sc->lanes = side_lanes();
            return e;
        }
        sc->lanes_open = true;
    }
    *out = sc;
    lane_bytes = arena_round(lane_bytes);
    shared_bytes = arena_round(shared_bytes);
    for (int n = sc->lanes.n; n >= 1; --n) {
        const size_t need = shared_bytes + (size_t)n * lane_bytes;
        if (sc->arena_bytes >= need) {
            *n_side = n;
            return hipSuccess;
        }
    }
    (void)hipStreamSynchronize(c->stream);
    if (sc->arena) {
        (void)hipFree(sc->arena);
        c->bytes -= (int64_t)sc->arena_bytes;
        sc->arena = nullptr;
        sc->arena_bytes = 0;
    }
    hipError_t e = hipErrorOutOfMemory;
    for (int n = sc->lanes.n; n >= 1; --n) {
        const size_t need = shared_bytes + (size_t)n * lane_bytes;
        e = hipMalloc((void **)&sc->arena, need);
        if (e == hipSuccess) {
            sc->arena_bytes = need;
            c->bytes += (int64_t)need;
            *n_side = n;
            return hipSuccess;
        }
        sc->arena = nullptr;
        (void)hipGetLastError();
    }
    return e;
}

// consecutive pieces of the arena
struct arena_cursor {
    char *p;
    template <class T>
    T *take(size_t count)
    {
        T *r = reinterpret_cast<T *>(p);
        p += arena_round(count * sizeof(T));
        return r;
    }
};

}  // namespace

void bagel_dgemm(hipStream_t st, int Mr, int Nc, int Kd, double alpha, const double *A, long sai, long sak,
                 const double *Bm, long sbk, long sbj, double *Cm, long ldc, bool overwrite)
{
    gemm(st, Mr, Nc, Kd, alpha, A, sai, sak, Bm, sbk, sbj, Cm, ldc, false, overwrite);
}

void bagel_release_setup(bagel_ctx *c)
{
    setup_scratch *sc = static_cast<setup_scratch *>(c->setup);
    if (!sc) return;
    sc->lanes.close();
    if (sc->arena) {
        (void)hipFree(sc->arena);
        c->bytes -= (int64_t)sc->arena_bytes;
    }
    delete sc;
    c->setup = nullptr;
}

int bagel_prepare_impl(bagel_ctx *c, const float *X, const float *y, const float *ell, const float *sf2,
                       const float *sn2, const float *omega, const float *phase, const float *w,
                       const float *eps, float *v_out)
{
    const int N = c->dm.N, L = c->dm.L, S = c->dm.S, M = c->M, D = c->D;
    const int Np = (N + NB - 1) / NB * NB;
    hipStream_t st = c->stream;
    setup_scratch *sc = nullptr;
    int n_side = 1;
    double *K[side_lanes::MAXL] = {}, *Phi[side_lanes::MAXL] = {}, *R[side_lanes::MAXL] = {}, *Wd[side_lanes::MAXL] = {};
    int *flag = nullptr;
    float h_sf2[8], h_sn2[8];
    int rc = BAGEL_OK;
    int h_flag = 0;

#define P_HIP(call)                                                                              \
    do {                                                                                         \
        hipError_t e__ = (call);                                                                 \
        if (e__ != hipSuccess) {                                                                 \
            snprintf(c->err, sizeof(c->err), "bagel_prepare_samples: %s failed: %s", #call,      \
                     hipGetErrorString(e__));                                                    \
            rc = (e__ == hipErrorOutOfMemory) ? BAGEL_ENOMEM : BAGEL_EHIP;                       \
            goto done;                                                                           \
        }                                                                                        \
    } while (0)

    {
        const size_t nK = (size_t)Np * Np, nPhi = (size_t)Np * L, nR = (size_t)Np * S, nW = (size_t)S * L;
        P_HIP(setup_reserve(c, M, arena_round(nK * 8) + arena_round(nPhi * 8) + arena_round(nR * 8) + arena_round(nW * 8),
                            sizeof(int), &sc, &n_side));
        arena_cursor cur{sc->arena};
        flag = cur.take<int>(1);
        for (int l = 0; l < n_side; ++l) {
            K[l] = cur.take<double>(nK);
            Phi[l] = cur.take<double>(nPhi);
            R[l] = cur.take<double>(nR);
            Wd[l] = cur.take<double>(nW);
        }
    }
    P_HIP(hipMemsetAsync(flag, 0, sizeof(int), st));
    P_HIP(hipMemcpyAsync(h_sf2, sf2, M * sizeof(float), hipMemcpyDeviceToHost, st));
    P_HIP(hipMemcpyAsync(h_sn2, sn2, M * sizeof(float), hipMemcpyDeviceToHost, st));
    P_HIP(hipStreamSynchronize(st));

    P_HIP(sc->lanes.fork(st));
    for (int m = 0; m < M; ++m) {
        const int l = m % n_side;
        hipStream_t ls = sc->lanes.st[l];
        hipLaunchKernelGGL(build_khat_kernel, dim3((Np + 255) / 256, Np), dim3(256), 0, ls, X, ell + (size_t)m * D,
                           h_sf2[m], h_sn2[m], K[l], N, Np, D);
        hipLaunchKernelGGL(build_phi_kernel, dim3((L + 255) / 256, Np), dim3(256), 0, ls, X,
                           omega + (size_t)m * L * D, phase + (size_t)m * L, h_sf2[m], Phi[l], N, Np, L, D);
        hipLaunchKernelGGL(init_rhs_kernel, dim3((S + 255) / 256, Np), dim3(256), 0, ls, y + (size_t)m * N, eps, R[l],
                           N, Np, S, M, m);
        // W of output m as float64 [S][L], so the GEMM reads one layout
        hipLaunchKernelGGL(convert_w_kernel, dim3((L + 255) / 256, S), dim3(256), 0, ls, w, Wd[l], S, M, L, m);
        // R -= Phi W^T : A = Phi [Np][L] (k fast), B(k=l, j=s) = Wd[s][l]
        gemm(ls, Np, S, L, -1.0, Phi[l], L, 1, Wd[l], 1, L, R[l], S, false);

        factor_and_solve(ls, K[l], Np, R[l], S, m * Np, flag);
        hipLaunchKernelGGL(emit_v_kernel, dim3((S + 255) / 256, c->Np / 4), dim3(256), 0, ls, R[l], v_out, c->v4, N,
                           c->Np, S, M, m);
        P_HIP(hipGetLastError());
    }
    P_HIP(sc->lanes.join(st));
    P_HIP(hipMemcpyAsync(&h_flag, flag, sizeof(int), hipMemcpyDeviceToHost, st));
    P_HIP(hipStreamSynchronize(st));
    if (h_flag != 0) {
        snprintf(c->err, sizeof(c->err),
                 "bagel_prepare_samples: K + noise_var I is not positive definite (output %d, pivot %d)",
                 (h_flag - 1) / Np, (h_flag - 1) % Np);
        rc = BAGEL_ENOTPD;
    }
done:
    if (sc) sc->lanes.sync();
    (void)hipStreamSynchronize(st);
    return rc;
#undef P_HIP
}

// Exact posterior cache of the per-step sampler (eq. (2), (3)): for every output alpha = K_hat^-1 y and
// K_hat^-1 itself, float64, padded to Np = multiple of 64 (the padding rows and columns of K_hat are an
// identity block, so they do not couple to the data; padded alpha entries are zero).
int bagel_prepare_posterior_impl(bagel_ctx *c, const float *X, const float *y, const float *ell, const float *sf2,
                                 const float *sn2)
{
    const int N = c->dm.N, M = c->M, D = c->D;
    const int Np = c->post_Np;
    hipStream_t st = c->stream;
    setup_scratch *sc = nullptr;
    int n_side = 1;
    double *K[side_lanes::MAXL] = {}, *Z[side_lanes::MAXL] = {}, *vec[side_lanes::MAXL] = {};
    int *flag = nullptr;
    float h_sf2[8], h_sn2[8];
    int rc = BAGEL_OK;
    int h_flag = 0;
#define P_HIP(call)                                                                              \
    do {                                                                                         \
        hipError_t e__ = (call);                                                                 \
        if (e__ != hipSuccess) {                                                                 \
            snprintf(c->err, sizeof(c->err), "bagel_prepare_posterior: %s failed: %s", #call,    \
                     hipGetErrorString(e__));                                                    \
            rc = (e__ == hipErrorOutOfMemory) ? BAGEL_ENOMEM : BAGEL_EHIP;                       \
            goto done;                                                                           \
        }                                                                                        \
    } while (0)
    {
        const size_t nK = (size_t)Np * Np;
        P_HIP(setup_reserve(c, M, 2 * arena_round(nK * 8) + arena_round((size_t)Np * 8), sizeof(int), &sc, &n_side));
        arena_cursor cur{sc->arena};
        flag = cur.take<int>(1);
        for (int l = 0; l < n_side; ++l) {
            K[l] = cur.take<double>(nK);
            Z[l] = cur.take<double>(nK);
            vec[l] = cur.take<double>(Np);
        }
    }
    P_HIP(hipMemsetAsync(flag, 0, sizeof(int), st));
    P_HIP(hipMemcpyAsync(h_sf2, sf2, M * sizeof(float), hipMemcpyDeviceToHost, st));
    P_HIP(hipMemcpyAsync(h_sn2, sn2, M * sizeof(float), hipMemcpyDeviceToHost, st));
    P_HIP(hipStreamSynchronize(st));
    P_HIP(sc->lanes.fork(st));
    for (int m = 0; m < M; ++m) {
        const int l = m % n_side;
        hipStream_t ls = sc->lanes.st[l];
        c->post_sf2[m] = (double)h_sf2[m];
        hipLaunchKernelGGL(build_khat_kernel, dim3((Np + 255) / 256, Np), dim3(256), 0, ls, X, ell + (size_t)m * D,
                           h_sf2[m], h_sn2[m], K[l], N, Np, D);
        inverse_from_factor(ls, K[l], Np, Z[l], y + (size_t)m * N, N, vec[l], c->post_Kinv + (size_t)m * Np * Np,
                            c->post_alpha + (size_t)m * Np, m * Np, flag);
        P_HIP(hipGetLastError());
    }
    P_HIP(sc->lanes.join(st));
    P_HIP(hipMemcpyAsync(&h_flag, flag, sizeof(int), hipMemcpyDeviceToHost, st));
    P_HIP(hipStreamSynchronize(st));
    if (h_flag != 0) {
        snprintf(c->err, sizeof(c->err),
                 "bagel_prepare_posterior: K + noise_var I is not positive definite (output %d, pivot %d)",
                 (h_flag - 1) / Np, (h_flag - 1) % Np);
        rc = BAGEL_ENOTPD;
    }
done:
    if (sc) sc->lanes.sync();
    (void)hipStreamSynchronize(st);
    return rc;
#undef P_HIP
}

// Log marginal likelihood of every output's GP and its gradient in the log hyper-parameters
// (eq. (5), (6)), n_iters > 0: Adam ascent on lml / N for n_iters iterations (Algorithm 1, "learn GP
// transition dynamics").  Buffers are allocated here and freed on return (set-up work).
int bagel_hyper_impl(bagel_ctx *c, const float *X, const float *y, float *log_hyp, float *lml, float *grad,
                     float *adam_m, float *adam_v, int n_iters, int first_step, double lr, double beta1, double beta2,
                     double eps)
{
    const int N = c->dm.N, M = c->M, D = c->D, H2 = c->D + 2;
    const int Np = (N + NB - 1) / NB * NB;
    hipStream_t st = c->stream;
    setup_scratch *sc = nullptr;
    int n_side = 1;
    double *K[side_lanes::MAXL] = {}, *Z[side_lanes::MAXL] = {}, *Kinv[side_lanes::MAXL] = {},
           *vec[side_lanes::MAXL] = {}, *partial[side_lanes::MAXL] = {};
    float *gneg = nullptr;
    int *flag = nullptr;
    int rc = BAGEL_OK, h_flag = 0;
#define P_HIP(call)                                                                              \
    do {                                                                                         \
        hipError_t e__ = (call);                                                                 \
        if (e__ != hipSuccess) {                                                                 \
            snprintf(c->err, sizeof(c->err), "bagel_hyper: %s failed: %s", #call, hipGetErrorString(e__)); \
            rc = (e__ == hipErrorOutOfMemory) ? BAGEL_ENOMEM : BAGEL_EHIP;                       \
            goto done;                                                                           \
        }                                                                                        \
    } while (0)
    {
        const size_t nK = (size_t)Np * Np;
        P_HIP(setup_reserve(c, M, 3 * arena_round(nK * 8) + arena_round((size_t)2 * Np * 8) + arena_round((size_t)N * H2 * 8),
                            arena_round(sizeof(int)) + arena_round((size_t)M * H2 * sizeof(float)), &sc, &n_side));
        arena_cursor cur{sc->arena};
        flag = cur.take<int>(1);
        gneg = cur.take<float>((size_t)M * H2);
        for (int l = 0; l < n_side; ++l) {
            K[l] = cur.take<double>(nK);
            Z[l] = cur.take<double>(nK);
            Kinv[l] = cur.take<double>(nK);
            vec[l] = cur.take<double>((size_t)2 * Np);          // y, alpha
            partial[l] = cur.take<double>((size_t)N * H2);
        }
    }
    P_HIP(hipMemsetAsync(flag, 0, sizeof(int), st));
    for (int it = 0; it < (n_iters > 0 ? n_iters : 1); ++it) {
        P_HIP(sc->lanes.fork(st));                      // after the parameter update of the previous iteration
        for (int m = 0; m < M; ++m) {
            const int l = m % n_side;
            hipStream_t ls = sc->lanes.st[l];
            const float *lh = log_hyp + (size_t)m * H2;
            hipLaunchKernelGGL(build_khat_log_kernel, dim3((Np + 255) / 256, Np), dim3(256), 0, ls, X, lh, K[l], N, Np, D);
            double *al = vec[l] + Np;
            inverse_from_factor(ls, K[l], Np, Z[l], y + (size_t)m * N, N, vec[l], Kinv[l], al, m * Np, flag);
            hipLaunchKernelGGL(hyper_lml_kernel, dim3(1), dim3(256), 0, ls, K[l], al, y + (size_t)m * N, N, Np,
                               lml + (size_t)it * M + m);
            hipLaunchKernelGGL(hyper_grad_rows_kernel, dim3(N), dim3(256), 0, ls, X, lh, Kinv[l], al, partial[l], N, Np, D);
            hipLaunchKernelGGL(hyper_grad_final_kernel, dim3(H2), dim3(256), 0, ls, partial[l], N, D,
                               grad ? grad + (size_t)m * H2 : nullptr, gneg + (size_t)m * H2);
            P_HIP(hipGetLastError());
        }
        P_HIP(sc->lanes.join(st));
        if (n_iters > 0) {
            const int step = first_step + it;
            P_HIP(bagel_launch_adam(c, log_hyp, gneg, adam_m, adam_v, M * H2, lr, beta1, beta2, eps,
                                    1.0 - pow(beta1, (double)step), 1.0 - pow(beta2, (double)step)));
        }
    }
    P_HIP(hipMemcpyAsync(&h_flag, flag, sizeof(int), hipMemcpyDeviceToHost, st));
    P_HIP(hipStreamSynchronize(st));
    if (h_flag != 0) {
        snprintf(c->err, sizeof(c->err), "bagel_hyper: K + noise_var I is not positive definite (output %d, pivot %d)",
                 (h_flag - 1) / Np, (h_flag - 1) % Np);
        rc = BAGEL_ENOTPD;
    }
done:
    if (sc) sc->lanes.sync();
    (void)hipStreamSynchronize(st);
    return rc;
#undef P_HIP
}
