// Policy network pi_theta([s ; g]): tanh MLP with a linear or saturating output (Sec. III-B and
// IV-A: feed-forward policy, bounded action), its backward pass, and the weight gradients.
//
// Forward / backward of one step: a workgroup holds 64 trajectories (lane = trajectory) and 16
// waves; each wave owns a contiguous group of output units of the current layer.  The layer's
// input activations live in LDS as [unit][lane] (conflict free), the weights are wave-uniform and
// arrive as scalar operands, so each LDS read feeds up to 16 FMAs.  Activations and adjoints are
// also written to the tape in HBM as [unit][B].
//
// Weight gradients are not accumulated inside the sweep: for each layer
//   dW[o][i] = sum_{t,b} delta[t][o][b] * h[t][i][b],   db[o] = sum_{t,b} delta[t][o][b]
// is one tall-skinny GEMM over the taped arrays with the contraction over (step, trajectory),
// computed with a fixed split of the contraction range and a fixed-order final sum, so the result
// is bitwise reproducible.
#include "bagel_internal.h"

namespace {

constexpr int PW = 16;   // waves per workgroup
constexpr int PL = 64;   // trajectories per workgroup

struct policy_args {
    int B, nl, ds;
    int width[4];
    int w_off[3], b_off[3];
    float act_bound;
    const float *W;       // forward: transposed weights [in][out]; backward: theta itself [out][in]
    float *h[3];          // tape slots of the layer inputs
    float *d[3];          // tape slots of the pre-activation adjoints
    float *a_slot;        // [d_a][B]
    float *dh0;           // [d_in][B]
    double *xbuf;         // [D][B]
};

// acc[jj] += sum_k Wk[k][j0+jj] * act[k][lane]; Wk is [nk][nj] row-major, j0 wave-uniform
template <int JPW>
__device__ __forceinline__ void dense(const float *__restrict__ Wk, int nk, int nj, int j0,
                                      const float *__restrict__ act, int lane, float *acc)
{
    for (int k = 0; k < nk; ++k) {
        const float hk = act[k * PL + lane];
        const float *__restrict__ row = Wk + (size_t)k * nj + j0;
#pragma unroll
        for (int jj = 0; jj < JPW; ++jj) acc[jj] = fmaf(row[jj], hk, acc[jj]);
    }
}

__device__ __forceinline__ void dense_dispatch(int jpw, const float *Wk, int nk, int nj, int j0,
                                               const float *act, int lane, float *acc)
{
    switch (jpw) {
        case 1: dense<1>(Wk, nk, nj, j0, act, lane, acc); break;
        case 2: dense<2>(Wk, nk, nj, j0, act, lane, acc); break;
        case 4: dense<4>(Wk, nk, nj, j0, act, lane, acc); break;
        case 8: dense<8>(Wk, nk, nj, j0, act, lane, acc); break;
        default: dense<16>(Wk, nk, nj, j0, act, lane, acc); break;
    }
}

// units per wave: smallest power of two p with 16 p >= nj
__device__ __host__ inline int units_per_wave(int nj)
{
    int p = 1;
    while (p * PW < nj) p *= 2;
    return p;
}

__global__ __launch_bounds__(PW * PL) void policy_forward_kernel(policy_args a)
{
    __shared__ float act[BAGEL_MAX_HIDDEN * PL];
    const int lane = threadIdx.x & (PL - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b_raw = blockIdx.x * PL + lane;
    const bool live = b_raw < a.B;
    const int b = live ? b_raw : a.B - 1;

    for (int k = wave; k < a.width[0]; k += PW) act[k * PL + lane] = a.h[0][(size_t)k * a.B + b];
    __syncthreads();

    for (int l = 0; l < a.nl; ++l) {
        const int nk = a.width[l], nj = a.width[l + 1];
        const int jpw = units_per_wave(nj);
        const int j0 = wave * jpw;
        float acc[16];
        const bool active = j0 < nj;    // nj is a multiple of jpw or smaller than 16 (jpw == 1)
        if (active) {
            const float *bias = a.W + a.b_off[l];
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) acc[jj] = (jj < jpw && j0 + jj < nj) ? bias[j0 + jj] : 0.0f;
            if (j0 + jpw <= nj) {
                dense_dispatch(jpw, a.W + a.w_off[l], nk, nj, j0, act, lane, acc);
            } else {
                // ragged last group: one unit at a time
                for (int jj = 0; j0 + jj < nj; ++jj) {
                    float s = acc[jj];
                    dense<1>(a.W + a.w_off[l], nk, nj, j0 + jj, act, lane, &s);
                    acc[jj] = s;
                }
            }
        }
        __syncthreads();
        if (active) {
            if (l < a.nl - 1) {
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    if (jj < jpw && j0 + jj < nj) {
                        const float hv = tanhf(acc[jj]);
                        act[(j0 + jj) * PL + lane] = hv;
                        if (live) a.h[l + 1][(size_t)(j0 + jj) * a.B + b] = hv;
                    }
                }
            } else {
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    if (jj < jpw && j0 + jj < nj && live) {
                        float out = acc[jj], act_v = acc[jj];
                        if (a.act_bound > 0.0f) {
                            act_v = tanhf(acc[jj]);
                            out = a.act_bound * act_v;
                        }
                        a.a_slot[(size_t)(j0 + jj) * a.B + b] = act_v;
                        a.xbuf[(size_t)(a.ds + j0 + jj) * a.B + b] = (double)out;
                    }
                }
            }
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(PW * PL) void policy_backward_kernel(policy_args a)
{
    __shared__ float act[BAGEL_MAX_HIDDEN * PL];
    const int lane = threadIdx.x & (PL - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b_raw = blockIdx.x * PL + lane;
    const bool live = b_raw < a.B;
    const int b = live ? b_raw : a.B - 1;

    const int last = a.nl - 1;
    for (int k = wave; k < a.width[a.nl]; k += PW) act[k * PL + lane] = a.d[last][(size_t)k * a.B + b];
    __syncthreads();

    for (int l = last; l >= 0; --l) {
        const int nk = a.width[l + 1], nj = a.width[l];   // contraction over outputs o, result per input i
        const int jpw = units_per_wave(nj);
        const int j0 = wave * jpw;
        float acc[16];
        const bool active = j0 < nj;
        if (active) {
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) acc[jj] = 0.0f;
            if (j0 + jpw <= nj) {
                dense_dispatch(jpw, a.W + a.w_off[l], nk, nj, j0, act, lane, acc);
            } else {
                for (int jj = 0; j0 + jj < nj; ++jj) {
                    float s = 0.0f;
                    dense<1>(a.W + a.w_off[l], nk, nj, j0 + jj, act, lane, &s);
                    acc[jj] = s;
                }
            }
        }
        __syncthreads();
        if (active) {
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                if (jj < jpw && j0 + jj < nj) {
                    const int j = j0 + jj;
                    if (l > 0) {
                        const float hv = a.h[l][(size_t)j * a.B + b];
                        const float dv = acc[jj] * (1.0f - hv * hv);
                        act[j * PL + lane] = dv;
                        if (live) a.d[l - 1][(size_t)j * a.B + b] = dv;
                    } else if (live) {
                        a.dh0[(size_t)j * a.B + b] = acc[jj];
                    }
                }
            }
        }
        __syncthreads();
    }
}

__global__ void transpose_theta_kernel(const float *__restrict__ theta, float *__restrict__ thetaT, int no,
                                       int ni, int w_off, int b_off)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < no * ni) {
        const int o = idx / ni, i = idx - o * ni;
        thetaT[w_off + i * no + o] = theta[w_off + idx];
    }
    if (idx < no) thetaT[b_off + idx] = theta[b_off + idx];
}

// ---- weight gradient GEMM ------------------------------------------------------------------
// C[o][i] = sum_k Dl[o][k] * Hl[i][k], k = (slot, b); column i == ni is the bias (Hl == 1).
// 64x64 tile per workgroup, 4x4 per thread, contraction in chunks of 32 staged through LDS.
constexpr int GT = 64, GK = 32;

__global__ __launch_bounds__(256) void weight_grad_kernel(const float *__restrict__ Dl, const float *__restrict__ Hl,
                                                          float *__restrict__ gsplit, int no, int ni, int B,
                                                          int n_slots, int chunks_per_slot, int chunks_per_split,
                                                          int w_off, int b_off, int P)
{
    __shared__ float As[GK][GT + 4];
    __shared__ float Bs[GK][GT + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int o0 = blockIdx.y * GT, i0 = blockIdx.x * GT;
    const int total_chunks = n_slots * chunks_per_slot;
    const int c_begin = blockIdx.z * chunks_per_split;
    const int c_end = min(total_chunks, c_begin + chunks_per_split);
    float acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int s = 0; s < 4; ++s) acc[r][s] = 0.0f;

    const int lr = tid >> 3;          // 0..31: row within the tile (and +32)
    const int lk = (tid & 7) * 4;     // k offset of this thread's 4 consecutive elements

    for (int c = c_begin; c < c_end; ++c) {
        const int slot = c / chunks_per_slot;
        const int kb = (c - slot * chunks_per_slot) * GK;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int r = lr + half * 32;
            const int o = o0 + r, i = i0 + r;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int bb = kb + lk + e;
                float av = 0.0f, bv = 0.0f;
                if (bb < B) {
                    if (o < no) av = Dl[((size_t)slot * no + o) * B + bb];
                    if (i < ni) bv = Hl[((size_t)slot * ni + i) * B + bb];
                    else if (i == ni) bv = 1.0f;
                }
                As[lk + e][r] = av;
                Bs[lk + e][r] = bv;
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < GK; ++k) {
            float av[4], bv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) av[r] = As[k][ty * 4 + r];
#pragma unroll
            for (int s = 0; s < 4; ++s) bv[s] = Bs[k][tx * 4 + s];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int s = 0; s < 4; ++s) acc[r][s] = fmaf(av[r], bv[s], acc[r][s]);
        }
        __syncthreads();
    }
    float *g = gsplit + (size_t)blockIdx.z * P;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int o = o0 + ty * 4 + r;
        if (o >= no) continue;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int i = i0 + tx * 4 + s;
            if (i < ni) g[w_off + (size_t)o * ni + i] = acc[r][s];
            else if (i == ni) g[b_off + o] = acc[r][s];
        }
    }
}

// gacc[p] (+)= sum_z gsplit[z][p] in z order; optionally emit grad_theta = (float) gacc
__global__ void grad_reduce_kernel(const float *__restrict__ gsplit, double *__restrict__ gacc, int P, int ksplit,
                                   bool accumulate, float *__restrict__ grad_theta)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    double s = accumulate ? gacc[p] : 0.0;
    for (int z = 0; z < ksplit; ++z) s += (double)gsplit[(size_t)z * P + p];
    gacc[p] = s;
    if (grad_theta) grad_theta[p] = (float)s;
}

policy_args make_pargs(const bagel_ctx *c, int slot)
{
    policy_args a;
    a.B = c->dm.B; a.nl = c->n_layers; a.ds = c->dm.d_s;
    for (int i = 0; i < 4; ++i) a.width[i] = c->width[i];
    for (int i = 0; i < 3; ++i) { a.w_off[i] = c->w_off[i]; a.b_off[i] = c->b_off[i]; }
    a.act_bound = c->dm.act_bound;
    const size_t B = c->dm.B;
    for (int l = 0; l < 3; ++l) {
        a.h[l] = (l < c->n_layers) ? c->tape_h[l] + (size_t)slot * c->width[l] * B : nullptr;
        a.d[l] = (l < c->n_layers && c->tape_d[l]) ? c->tape_d[l] + (size_t)slot * c->width[l + 1] * B : nullptr;
    }
    a.a_slot = c->tape_a + (size_t)slot * c->dm.d_a * B;
    a.dh0 = c->dh0;
    a.xbuf = c->xbuf;
    a.W = nullptr;
    return a;
}

}  // namespace

hipError_t bagel_launch_transpose_theta(bagel_ctx *c, const float *theta)
{
    for (int l = 0; l < c->n_layers; ++l) {
        const int no = c->width[l + 1], ni = c->width[l];
        hipLaunchKernelGGL(transpose_theta_kernel, dim3((no * ni + 255) / 256), dim3(256), 0, c->stream, theta,
                           c->thetaT, no, ni, c->w_off[l], c->b_off[l]);
    }
    return hipGetLastError();
}

hipError_t bagel_launch_policy_forward(bagel_ctx *c, int slot)
{
    policy_args a = make_pargs(c, slot);
    a.W = c->thetaT;
    hipLaunchKernelGGL(policy_forward_kernel, dim3((c->dm.B + PL - 1) / PL), dim3(PW * PL), 0, c->stream, a);
    return hipGetLastError();
}

hipError_t bagel_launch_policy_backward(bagel_ctx *c, int slot, const float *theta)
{
    policy_args a = make_pargs(c, slot);
    a.W = theta;
    hipLaunchKernelGGL(policy_backward_kernel, dim3((c->dm.B + PL - 1) / PL), dim3(PW * PL), 0, c->stream, a);
    return hipGetLastError();
}

hipError_t bagel_launch_weight_grad(bagel_ctx *c, int n_slots, bool accumulate, float *grad_theta)
{
    const int B = c->dm.B;
    const int chunks_per_slot = (B + GK - 1) / GK;
    const int total = n_slots * chunks_per_slot;
    const int ksplit = total < c->ksplit ? total : c->ksplit;
    const int per = (total + ksplit - 1) / ksplit;
    const int nz = (total + per - 1) / per;
    for (int l = 0; l < c->n_layers; ++l) {
        const int no = c->width[l + 1], ni = c->width[l];
        dim3 grid((ni + 1 + GT - 1) / GT, (no + GT - 1) / GT, nz);
        hipLaunchKernelGGL(weight_grad_kernel, grid, dim3(256), 0, c->stream, c->tape_d[l], c->tape_h[l], c->gsplit, no,
                           ni, B, n_slots, chunks_per_slot, per, c->w_off[l], c->b_off[l], c->P);
    }
    hipLaunchKernelGGL(grad_reduce_kernel, dim3((c->P + 255) / 256), dim3(256), 0, c->stream, c->gsplit, c->gacc, c->P,
                       nz, accumulate, grad_theta);
    return hipGetLastError();
}
