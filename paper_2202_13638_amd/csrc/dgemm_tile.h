// Tile routine of the float64 matrix products: C[i][j] (+)= alpha * sum_k A(i,k) B(k,j) with
// A(i,k) = A[i*sai + k*sak], B(k,j) = B[k*sbk + j*sbj].
// A workgroup of 256 threads owns a 64 x 64 tile of the result; its four waves own 32 x 32 quarters
// as 2 x 2 tiles of v_mfma_f64_16x16x4 (D[16x16] += A[16x4] B[4x16]; lane l feeds A[i = l % 16][k = l / 16]
// and B[k = l / 16][j = l % 16]; register r of lane l holds D[row = l / 16 + 4 r][col = l % 16]).
// Operand tiles of 16 contraction indices go through LDS as [k][i] with rows padded by one element,
// so the 16 lanes of a k-row read consecutive addresses; the next operand tiles are fetched into
// registers under the MFMAs.  The float64 matrix pipe has the rate of the vector pipe on this chip, but
// it needs one LDS read per 512 FMAs where a vector-FMA micro-tile needs one per 2.  (A 128 x 128
// tile was measured too: no faster on the [2048 x 2048] x [2048 x 1024] products of the posterior
// sampler, where it leaves half the compute units without a tile, and slower on the 64-deep updates of
// the blocked factorisation.)
// What happens to the finished tile is the caller's: the epilogue receives the wave's accumulators.
#pragma once
#include <hip/hip_runtime.h>

namespace bagel_gemm {

constexpr int TM = 64, TN = 64, TK = 16;
typedef double d4v __attribute__((ext_vector_type(4)));

struct tile_lds {
    double As[TK][TM + 1];
    double Bs[TK][TN + 1];
};

// Position of a lane's accumulator entries inside the 64 x 64 tile: entry acc[x][y][r] is element
// (row0 + 16 x + 4 r, col0 + 16 y) of the tile.
struct lane_pos {
    int row0, col0;
};

__device__ __forceinline__ lane_pos lane_position()
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    return lane_pos{(wave >> 1) * 32 + (lane >> 4), (wave & 1) * 32 + (lane & 15)};
}

// acc = sum_k A(i0 + i, k) B(k, j0 + j) over k in [0, Kd) for the workgroup's tile; elements outside
// [0, Mr) x [0, Nc) x [0, Kd) count as zero.  Ends with a barrier: the LDS tiles may be reused.
__device__ __forceinline__ void tile_product(d4v (&acc)[2][2], tile_lds &sh, int i0, int j0, int Mr, int Nc, int Kd,
                                             const double *__restrict__ A, long sai, long sak,
                                             const double *__restrict__ Bm, long sbk, long sbj)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wi = (wave >> 1) * 32, wj = (wave & 1) * 32;     // the wave's quarter of the tile
    const int lr = lane & 15, lk = lane >> 4;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] = d4v{0.0, 0.0, 0.0, 0.0};
    // loaders: pick the thread->element map that walks the unit-stride direction fastest
    const bool a_k_fast = (sak == 1);
    const bool b_j_fast = (sbj == 1);
    constexpr int PER = TM * TK / 256;                // elements of each operand tile per thread
    double ra[PER], rb[PER];
    auto fetch = [&](int k0) {                        // global -> registers (zero outside the matrices)
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const int idx = tid + e * 256;
            int ii, kk;
            if (a_k_fast) { kk = idx % TK; ii = idx / TK; } else { ii = idx % TM; kk = idx / TM; }
            const int gi = i0 + ii, gk = k0 + kk;
            ra[e] = (gi < Mr && gk < Kd) ? A[(long)gi * sai + (long)gk * sak] : 0.0;
            int jj, kb;
            if (b_j_fast) { jj = idx % TN; kb = idx / TN; } else { kb = idx % TK; jj = idx / TK; }
            const int gj = j0 + jj, gkb = k0 + kb;
            rb[e] = (gj < Nc && gkb < Kd) ? Bm[(long)gkb * sbk + (long)gj * sbj] : 0.0;
        }
    };
    auto stash = [&]() {                              // registers -> LDS
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const int idx = tid + e * 256;
            int ii, kk;
            if (a_k_fast) { kk = idx % TK; ii = idx / TK; } else { ii = idx % TM; kk = idx / TM; }
            sh.As[kk][ii] = ra[e];
            int jj, kb;
            if (b_j_fast) { jj = idx % TN; kb = idx / TN; } else { kb = idx % TK; jj = idx / TK; }
            sh.Bs[kb][jj] = rb[e];
        }
    };
    fetch(0);
    stash();
    __syncthreads();
    for (int k0 = 0; k0 < Kd; k0 += TK) {
        const bool more = k0 + TK < Kd;
        if (more) fetch(k0 + TK);                     // in flight under the MFMAs below
#pragma unroll
        for (int ks = 0; ks < TK; ks += 4) {
            double av[2], bv[2];
#pragma unroll
            for (int x = 0; x < 2; ++x) av[x] = sh.As[ks + lk][wi + 16 * x + lr];
#pragma unroll
            for (int y = 0; y < 2; ++y) bv[y] = sh.Bs[ks + lk][wj + 16 * y + lr];
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y)
                    acc[x][y] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[x], bv[y], acc[x][y], 0, 0, 0);
        }
        __syncthreads();
        if (more) stash();
        __syncthreads();
    }
}

}  // namespace bagel_gemm
