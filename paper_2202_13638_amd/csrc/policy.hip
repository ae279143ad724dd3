// Policy network pi_theta([s ; g]): tanh MLP with a linear or saturating output (Sec. III-B and
// IV-A: feed-forward policy, bounded action), the end of a rollout step around it, the backward
// sweep of Algorithm 1, the weight gradients and the Adam update.  The layers are dense float32
// contractions and run on the matrix cores (v_mfma_f32_32x32x2_f32: D[32x32] += A[32x2] B[2x32]).
//
// Layers, forward and backward.  A workgroup holds 32 trajectories and 8 waves; a wave owns the
// 32x32 output tile of units [32 rt, 32 rt + 32) x the 32 trajectories (and, when a layer has fewer
// than 8 row tiles, one slice of the contraction; slices are added through LDS in a fixed order).
//   A operand = weights, zero-padded to [rows % 32 == 0][K % 32 == 0] and re-ordered once per call
//               so that a wave reads the operands of four MFMAs as 1 KB of contiguous memory; the
//               forward kernels keep the wave's share of all layers in registers, the backward
//               sweep keeps the two narrow layers there and streams the wide one from L2 one batch
//               of 16 MFMAs ahead;
//   B operand = the layer's input activations, kept in LDS as [K/4][trajectory][4] so a lane
//               reads the matching four K values of its trajectory with one 16-byte load.
// Lanes 0-31 feed K = k0..k0+3 and lanes 32-63 feed K = k0+4..k0+7 over four MFMAs; the order in
// which K is consumed does not matter as long as A and B agree.  The epilogue (bias, tanh, or the
// tanh derivative in the backward pass) writes the next layer's input back to LDS in the same
// layout and to the tape in HBM as [unit][B].
//
// Kernels: policy_forward_kernel (first step of a rollout or segment), step_tail_kernel (everything
// between two sample evaluations: reduction of the partial sums, state update, cost, tapes, policy
// of the next step), backward_sweep_kernel (all backward steps of a tape segment in one launch).
//
// Weight gradients are not accumulated inside the sweep.  For each layer
//   dW[o][i] = sum_{t,b} delta[t][o][b] * h[t][i][b],   db[o] = sum_{t,b} delta[t][o][b]
// is one GEMM over the taped arrays with the contraction over (step, trajectory): operands staged
// through LDS for the wide layer (weight_grad_tiled_kernel), read straight from the tape for the
// narrow ones (weight_grad_kernel).  The contraction range is split over workgroups in a fixed way
// and the partial results are added in a fixed order, so the gradient is bitwise reproducible.
#include "bagel_internal.h"
#include <type_traits>

namespace {

typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int PW = 8;    // waves per workgroup
constexpr int PL = 32;   // trajectories per workgroup

struct policy_args {
    int B, nl, ds;
    int width[4];
    int b_off[3];         // bias offsets inside theta
    int wp_off[3];        // offsets of the packed weight matrices
    int kp[3], rp[3];     // padded contraction length and row count per layer
    float act_bound;
    const float *theta;
    const float *Wp;      // packed forward weights (rows = outputs)
    float *h[3];          // tape slots of the layer inputs
    float *a_slot;        // [d_a][B]
    double *xbuf;         // [D][B]
};

// How the 8 waves share a layer with `rows` output rows and padded contraction length kp: wave =
// ks * nrt + rt owns row tile rt and the ks-th slice of the contraction.  Layers with fewer than 8
// row tiles split the contraction instead of idling waves.
struct wave_plan {
    int nrt, ksplit, rt, ks, k_begin, k_end;
    bool active;
};

__device__ __forceinline__ wave_plan plan_layer(int rows, int kp, int wave)
{
    wave_plan p;
    p.nrt = (rows + 31) >> 5;
    p.ksplit = PW / p.nrt;
    if (p.ksplit < 1) p.ksplit = 1;
    const int k32 = kp >> 5;                      // contraction length in batches of 32 (kp % 32 == 0)
    if (p.ksplit > k32) p.ksplit = k32;
    p.rt = wave % p.nrt;
    p.ks = wave / p.nrt;
    p.active = p.ks < p.ksplit;
    const int per = (k32 + p.ksplit - 1) / p.ksplit;
    p.k_begin = 4 * p.ks * per;                   // in groups of 8, always a multiple of 4
    p.k_end = p.k_begin + 4 * per < 4 * k32 ? p.k_begin + 4 * per : 4 * k32;
    return p;
}

// 16-byte read that the optimiser will not move across loop iterations (two relaxed wave-scope
// atomic loads: an ordinary load instruction, but one the compiler keeps where it is written).
// Used to keep the look-ahead operand loads of the MFMA loops ahead of the MFMAs; plain loads of
// read-only memory are sunk back next to their use, which exposes the full memory latency.
__device__ __forceinline__ float4 load16_pinned(const float4 *p)
{
    const unsigned long long *q = reinterpret_cast<const unsigned long long *>(p);
    const unsigned long long lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    const unsigned long long hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    float4 r;
    r.x = __uint_as_float((unsigned)lo);
    r.y = __uint_as_float((unsigned)(lo >> 32));
    r.z = __uint_as_float((unsigned)hi);
    r.w = __uint_as_float((unsigned)(hi >> 32));
    return r;
}

__device__ __forceinline__ f16v mfma_batch(f16v acc, const float4 *av, const float4 *bv)
{
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u].x, bv[u].x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u].y, bv[u].y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u].z, bv[u].z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u].w, bv[u].w, acc, 0, 0, 0);
    }
    return acc;
}

// acc = W[32 rt .. +32][8 k_begin .. 8 k_end) * act[same K][32 trajectories].
// Packed weights: element W[32 rt + c][8 k8 + 4 hf + e] sits at ((rt * kp/8 + k8) * 64 + c + 32 hf) * 4 + e,
// so a wave reads 1 KB contiguous per 8 values of K.  The contraction is consumed in batches of 32
// (16 MFMAs); the weight fragments of the next batch are requested before the MFMAs of the current
// one issue.  All loads are unconditional (kp is padded to a multiple of 32 with zero weights; the
// look-ahead past the end re-reads the last batch).
__device__ __forceinline__ f16v tile_contract(const float *__restrict__ W, int kp, const wave_plan &p, int lane,
                                              const float4 *__restrict__ act4)
{
    f16v acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
    if (p.k_begin >= p.k_end) return acc;
    const int c = lane & 31, hf = lane >> 5;
    const float4 *wfrag = reinterpret_cast<const float4 *>(W) + (size_t)p.rt * (kp >> 3) * 64 + lane;
    const float4 *bcol = act4 + hf * PL + c;
    float4 a0[4], a1[4], bv[4];      // two weight batches in turn: one feeding MFMAs, one in flight
#pragma unroll
    for (int u = 0; u < 4; ++u) a0[u] = load16_pinned(wfrag + (size_t)(p.k_begin + u) * 64);
    for (int k8 = p.k_begin;; k8 += 8) {
        const bool more1 = k8 + 4 < p.k_end;            // wave-uniform
        if (more1) {
#pragma unroll
            for (int u = 0; u < 4; ++u) a1[u] = load16_pinned(wfrag + (size_t)(k8 + 4 + u) * 64);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) bv[u] = bcol[((k8 + u) * 2) * PL];
        acc = mfma_batch(acc, a0, bv);
        if (!more1) break;
        const bool more2 = k8 + 8 < p.k_end;
        if (more2) {
#pragma unroll
            for (int u = 0; u < 4; ++u) a0[u] = load16_pinned(wfrag + (size_t)(k8 + 8 + u) * 64);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) bv[u] = bcol[((k8 + 4 + u) * 2) * PL];
        acc = mfma_batch(acc, a1, bv);
        if (!more2) break;
    }
    return acc;
}

// The weights a wave multiplies with are read once per launch and stay in its registers.
// Packed weights: element W[32 rt + c][8 k8 + 4 hf + e] sits at ((rt * kp/8 + k8) * 64 + c + 32 hf) * 4 + e,
// so a "group" (8 contraction indices) is one float4 per lane and a wave reads it as 1 KB of
// contiguous memory.  A wave's slice of a layer, groups [k_begin, k_end), is a whole number of
// batches of 4 groups (kp is a multiple of 32) and at most 8 batches (a 32 x 256 block).
template <int NBMAX>
__device__ __forceinline__ void load_wave_weights(float4 (&w)[4 * NBMAX], const float *__restrict__ W, int kp,
                                                  const wave_plan &p, int lane)
{
    if (!p.active) return;
    const float4 *wfrag = reinterpret_cast<const float4 *>(W) + ((size_t)p.rt * (kp >> 3) + p.k_begin) * 64 + lane;
    const int nb = (p.k_end - p.k_begin) >> 2;
#pragma unroll
    for (int ub = 0; ub < NBMAX; ++ub)
        if (ub < nb) {
#pragma unroll
            for (int u = 0; u < 4; ++u) w[4 * ub + u] = wfrag[(size_t)(4 * ub + u) * 64];
        }
}

__device__ __forceinline__ f16v mfma_group(f16v acc, const float4 av, const float4 bv)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.x, bv.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.y, bv.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.z, bv.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.w, bv.w, acc, 0, 0, 0);
    return acc;
}

// acc = W[wave's rows][its slice of the contraction] * act[same K][32 trajectories]: weights from
// registers, activations from LDS as [K/4][trajectory][4], one batch (4 groups, 16 MFMAs) at a time.
template <int NBMAX>
__device__ __forceinline__ f16v contract_batches(const float4 (&w)[4 * NBMAX], const wave_plan &p, int lane,
                                                 const float4 *__restrict__ act4)
{
    f16v acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
    const float4 *bcol = act4 + ((size_t)p.k_begin * 2 + (lane >> 5)) * PL + (lane & 31);
    const int nb = (p.k_end - p.k_begin) >> 2;
#pragma unroll
    for (int ub = 0; ub < NBMAX; ++ub)
        if (ub < nb) {
            float4 bv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) bv[u] = bcol[(4 * ub + u) * 2 * PL];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = mfma_group(acc, w[4 * ub + u], bv[u]);
        }
    return acc;
}

// Add the partial tiles of the other contraction slices (through LDS, fixed order).  Contains the
// barrier that also separates the reads of the layer input from the writes of the next one.
__device__ __forceinline__ void combine_slices(f16v &acc, const wave_plan &p, int wave, int lane, float4 *red4)
{
    if (p.ksplit > 1 && p.active && p.ks > 0) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
            red4[(wave * 4 + g) * 64 + lane] = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
    }
    __syncthreads();
    if (p.ksplit > 1 && p.active && p.ks == 0) {
        for (int s = 1; s < p.ksplit; ++s) {
            const int w = s * p.nrt + p.rt;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 t = red4[(w * 4 + g) * 64 + lane];
                acc[4 * g] += t.x; acc[4 * g + 1] += t.y; acc[4 * g + 2] += t.z; acc[4 * g + 3] += t.w;
            }
        }
    }
}

// tanh in float32 from the hardware exp2 and reciprocal: 1 - 2 / (e^{2z} + 1), five instructions
// (e^{2z} overflows to +inf for large z, where the reciprocal gives 0, and underflows to 0 for very
// negative z: both ends come out as +-1 without a case distinction).  Absolute error below 2.5e-7 over the
// whole range; a fraction of the instructions of the library routine, which matters because a layer's
// epilogue evaluates 8192 of them per workgroup and is bound by instruction issue.  (A form with a
// polynomial branch below |z| = 1/4 kept the relative error small near zero as well, at three times the
// instructions; what the next layer and the tanh derivative see is the absolute error.)
__device__ __forceinline__ float tanh_fast(float z)
{
    const float t = __builtin_amdgcn_exp2f(z * 2.8853900817779268f);           // e^{2z}
    return fmaf(-2.0f, __builtin_amdgcn_rcpf(t + 1.0f), 1.0f);
}

// rows of a [n][B] array -> LDS [k/4][trajectory][4], zero-filled up to kp rows
__device__ __forceinline__ void stage_input(const float *__restrict__ src, int n, int kp, int B, int b0,
                                            float4 *__restrict__ act4)
{
    const int bl = threadIdx.x & (PL - 1);
    int b = b0 + bl;
    if (b >= B) b = B - 1;
    for (int kg = threadIdx.x / PL; kg < (kp >> 2); kg += PW * 64 / PL) {
        float t[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int k = kg * 4 + e;
            t[e] = k < n ? src[(size_t)k * B + b] : 0.0f;
        }
        act4[kg * PL + bl] = make_float4(t[0], t[1], t[2], t[3]);
    }
}

// Per-wave register copy of the forward weights (requested first in a kernel: they arrive while the
// layer-0 input is being produced), the share of each layer the wave works on, and the biases in LDS.
// The three arrays are separate locals of the calling kernel so that they are promoted to registers.
#define FORWARD_WEIGHTS_DECL                                   \
    float4 w_first[4], w_last[4], w_wide[32];                  \
    float bias_r[3];                                           \
    wave_plan p_first, p_last, p_wide

__device__ __forceinline__ void load_forward_weights(const policy_args &a, int wave, int lane, float4 (&w_first)[4],
                                                     float4 (&w_last)[4], float4 (&w_wide)[32], wave_plan &p_first,
                                                     wave_plan &p_last, wave_plan &p_wide, float (&bias_r)[3])
{
    p_first = plan_layer(a.width[1], a.kp[0], wave);
    p_last = plan_layer(a.width[a.nl], a.kp[a.nl - 1], wave);
    p_wide = p_first;
    load_wave_weights<1>(w_first, a.Wp + a.wp_off[0], a.kp[0], p_first, lane);
    if (a.nl == 3) {
        p_wide = plan_layer(a.width[2], a.kp[1], wave);
        load_wave_weights<8>(w_wide, a.Wp + a.wp_off[1], a.kp[1], p_wide, lane);
    }
    load_wave_weights<1>(w_last, a.Wp + a.wp_off[a.nl - 1], a.kp[a.nl - 1], p_last, lane);
    // biases: one value per thread and layer (a layer is at most 256 wide), parked in registers; writing
    // them to LDS right away would wait for every load requested above
#pragma unroll
    for (int l = 0; l < 3; ++l)
        bias_r[l] = (l < a.nl && (int)threadIdx.x < a.width[l + 1]) ? a.theta[a.b_off[l] + threadIdx.x] : 0.0f;
}

// second half of load_forward_weights, to be called once the loads have had time to arrive
__device__ __forceinline__ void stash_biases(const policy_args &a, const float (&bias_r)[3],
                                             float (*biasS)[BAGEL_MAX_HIDDEN])
{
#pragma unroll
    for (int l = 0; l < 3; ++l)
        if (l < a.nl && (int)threadIdx.x < a.width[l + 1]) biasS[l][threadIdx.x] = bias_r[l];
}

// Element at a wave-uniform base plus a 32-bit byte offset per lane: the form in which the address costs no
// vector arithmetic (the base stays in scalar registers and is advanced there).
__device__ __forceinline__ float *at_byte(float *base, unsigned byte_off)
{
    return reinterpret_cast<float *>(reinterpret_cast<char *>(base) + byte_off);
}

// Bias, activation, tape and next-layer input for the four consecutive output units row_u + 4 hf + (0..3)
// of layer l (row_u: wave-uniform, a multiple of 8) and trajectory column c of the workgroup (z4: the
// contraction results).  An epilogue is bound by instruction issue (8192 activations per workgroup and
// 256-unit layer), so the tape addresses are a scalar row base plus one lane offset, and the four biases
// come as one LDS read.
__device__ __forceinline__ void layer_epilogue(const policy_args &a, size_t slot, bool write_x, int l, int row_u, int hf,
                                               int c, int b0, const float (&z4)[4], const float *bias, float4 *act4)
{
    const int nj = a.width[l + 1];
    const int b = b0 + c;
    const bool live = b < a.B;
    const int jb = row_u + 4 * hf;
    const unsigned lane_off = ((unsigned)(4 * hf) * (unsigned)a.B + (unsigned)b) * 4u;
    const float4 bias4 = *reinterpret_cast<const float4 *>(bias + jb);      // entries past nj are not used
    const float bz[4] = {bias4.x, bias4.y, bias4.z, bias4.w};
    float out[4];
    if (l < a.nl - 1) {
        float *hrow = a.h[l + 1] + (slot * nj + row_u) * a.B;              // wave-uniform
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool on = jb + e < nj;
            const float hv = on ? tanh_fast(z4[e] + bz[e]) : 0.0f;
            out[e] = hv;
            if (live && on) *at_byte(hrow + (size_t)e * a.B, lane_off) = hv;
        }
        act4[(jb >> 2) * PL + c] = make_float4(out[0], out[1], out[2], out[3]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = jb + e;
            if (live && j < nj) {
                const float z = z4[e] + bz[e];
                float act_v = z, act_out = z;
                if (a.act_bound > 0.0f) {
                    act_v = tanh_fast(z);
                    act_out = a.act_bound * act_v;
                }
                a.a_slot[(slot * nj + j) * a.B + b] = act_v;
                if (write_x) a.xbuf[(size_t)(a.ds + j) * a.B + b] = (double)act_out;
            }
        }
    }
}

// The layers of pi_theta for the 32 trajectories of a workgroup, input in act4 (all waves past a
// barrier after it was written).  Writes the tape (h of the hidden layers, the action before
// scaling; `slot` counts tape slots from the ones a.h and a.a_slot point at) and, with write_x, the
// action into xbuf.
// A layer whose contraction is not split (8 row tiles: 256 units) finishes in the registers of the wave
// that owns the tile.  A narrower layer splits the contraction over the waves; there every slice goes
// to LDS and the sums, in slice order, and the epilogue are spread over all 512 threads (four units of
// one trajectory each): with two row tiles the epilogue of a layer is 4 activations per thread
// instead of 16 on two of the eight waves, and it is the epilogues, not the matrix instructions, that
// a narrow policy's step spends its time on.
__device__ __forceinline__ void policy_layers(const policy_args &a, const float4 (&w_first)[4],
                                              const float4 (&w_last)[4], const float4 (&w_wide)[32],
                                              const wave_plan &p_first, const wave_plan &p_last,
                                              const wave_plan &p_wide, int wave, int lane, int b0, float4 *act4,
                                              float4 *red4, const float (*biasS)[BAGEL_MAX_HIDDEN], size_t slot = 0,
                                              bool write_x = true)
{
    const int c = lane & 31, hf = lane >> 5;
    for (int l = 0; l < a.nl; ++l) {
        const wave_plan p = l == 0 ? p_first : (l == a.nl - 1 ? p_last : p_wide);
        f16v acc;
        if (p.active) {
            if (l == 0) acc = contract_batches<1>(w_first, p, lane, act4);
            else if (l == a.nl - 1) acc = contract_batches<1>(w_last, p, lane, act4);
            else acc = contract_batches<8>(w_wide, p, lane, act4);
        }
        if (p.ksplit == 1) {
            __syncthreads();                 // every wave has read the layer input: act4 may be rewritten
            if (p.active) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float z4[4] = {acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
                    layer_epilogue(a, slot, write_x, l, p.rt * 32 + 8 * g, hf, c, b0, z4, biasS[l], act4);
                }
            }
        } else {
            if (p.active) {
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    red4[(wave * 4 + g) * 64 + lane] = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
            }
            __syncthreads();
            // item = (row tile, register group g, lane) of a tile: 256 per row tile, at most 7 row tiles here
            for (int item = threadIdx.x; item < p.nrt * 256; item += PW * 64) {
                const int iw = __builtin_amdgcn_readfirstlane(item >> 6);     // the same for all lanes of a wave
                const int rt = iw >> 2, g = iw & 3, ln = item & 63;
                float4 t = red4[((0 * p.nrt + rt) * 4 + g) * 64 + ln];
                for (int sl = 1; sl < p.ksplit; ++sl) {
                    const float4 u = red4[((sl * p.nrt + rt) * 4 + g) * 64 + ln];
                    t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
                }
                const float z4[4] = {t.x, t.y, t.z, t.w};
                layer_epilogue(a, slot, write_x, l, rt * 32 + 8 * g, ln >> 5, ln & 31, b0, z4, biasS[l], act4);
            }
        }
        __syncthreads();
    }
}

// Policy of one step on its own (first step of a rollout or of a replayed segment): input from tape slot h[0].
__global__ __launch_bounds__(PW * 64) void policy_forward_kernel(policy_args a)
{
    __shared__ float4 act4[(BAGEL_MAX_HIDDEN / 4) * PL];   // layer input  [K/4][trajectory]
    __shared__ float4 red4[PW * 4 * 64];                   // partial tiles of split contractions
    __shared__ __align__(16) float biasS[3][BAGEL_MAX_HIDDEN];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b0 = blockIdx.x * PL;
    FORWARD_WEIGHTS_DECL;
    load_forward_weights(a, wave, lane, w_first, w_last, w_wide, p_first, p_last, p_wide, bias_r);
    stage_input(a.h[0], a.width[0], a.kp[0], a.B, b0, act4);
    stash_biases(a, bias_r, biasS);
    __syncthreads();
    policy_layers(a, w_first, w_last, w_wide, p_first, p_last, p_wide, wave, lane, b0, act4, red4, biasS);
}

// Policy of the steps t0 .. t0 + n_slots - 1 at once, from the kept states: rebuilds the activation
// tape of a segment (gradient checkpointing, Sec. IV-C).  Tape slot = t - t0; the input
// [s_t ; g_t] is the float32 state of the tape, the same numbers the forward pass fed to the policy,
// so the activations come out bit for bit as they were.  Nothing is written to xbuf.
struct replay_args {
    const float *tape_s;      // [H+1][d_s][B]
    const float *goals;       // [H][B][d_g]
    int t0, dg, n_slots;
};
constexpr int REPLAY_SLOTS = 5;   // steps per workgroup

__global__ __launch_bounds__(PW * 64) void policy_replay_kernel(policy_args a, replay_args r)
{
    __shared__ float4 act4[(BAGEL_MAX_HIDDEN / 4) * PL];
    __shared__ float4 red4[PW * 4 * 64];
    __shared__ __align__(16) float biasS[3][BAGEL_MAX_HIDDEN];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b0 = blockIdx.x * PL;
    const size_t B = a.B;
    FORWARD_WEIGHTS_DECL;
    load_forward_weights(a, wave, lane, w_first, w_last, w_wide, p_first, p_last, p_wide, bias_r);
    stash_biases(a, bias_r, biasS);
    // A workgroup keeps the weights in its registers for REPLAY_SLOTS consecutive steps: fetching them
    // is what a replay launch spends most of its time on when every step has workgroups of its own.
    const int s_begin = blockIdx.y * REPLAY_SLOTS;
    const int s_end = min(r.n_slots, s_begin + REPLAY_SLOTS);
    for (int sl = s_begin; sl < s_end; ++sl) {
        const size_t slot = (size_t)sl;
        const int t = r.t0 + sl;
        {   // layer-0 input from the state tape and the goals, to LDS and to its tape slot
            const int bl = threadIdx.x & (PL - 1);
            const bool live = b0 + bl < a.B;
            const int b = live ? b0 + bl : a.B - 1;
            for (int kg = threadIdx.x / PL; kg < (a.kp[0] >> 2); kg += PW * 64 / PL) {
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = kg * 4 + e;
                    v[e] = 0.0f;
                    if (k < a.ds) v[e] = r.tape_s[((size_t)t * a.ds + k) * B + b];
                    else if (k < a.ds + r.dg) v[e] = r.goals[((size_t)t * B + b) * r.dg + (k - a.ds)];
                    if (live && k < a.ds + r.dg) a.h[0][(slot * a.width[0] + k) * B + b] = v[e];
                }
                act4[kg * PL + bl] = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
        __syncthreads();
        // ends with a barrier: act4 may be rewritten for the next slot
        policy_layers(a, w_first, w_last, w_wide, p_first, p_last, p_wide, wave, lane, b0, act4, red4, biasS, slot, false);
    }
}

// ---- end of step t and policy of step t+1 in one launch -------------------------------------
// After the sample evaluation of step t: add up the value sums of its work units (f; the Jacobian sums
// are added up off the critical path, see gp_step.hip), advance the state s_{t+1} = s_t + f (state
// increments as GP targets, Sec. III-A), add the cost of s_{t+1} against the goal of step t (Algorithm 1,
// return accumulation), write the state tape, and - unless this was the last step - run
// pi_theta([s_{t+1} ; g_{t+1}]) for the same 32 trajectories straight from LDS.  The weights are
// requested before the reduction starts.  The state is read from one input buffer and written, with the
// new action, to the other (the caller swaps them), so that the inputs of step t stay intact for the
// deferred Jacobian sums.
struct tail_args {
    int D, M, dg, ngk, ngl, ncomp;      // ncomp = 1 (value only) or 1 + D (with Jacobian)
    int cost_kind, add_cost, do_policy;
    int direct;                         // part holds f and J_f themselves, [m][1+D][B] (per-step posterior sampler)
    float sigma_r;
    int tracked[8];
    float q[8];
    const double *A, *amp, *part;       // part: [groups][1+D][B]
    const double *x_cur;                // [D][B] inputs of step t (rows < d_s: s_t)
    double *x_next;                     // [D][B] receives s_{t+1} (the policy adds a_{t+1})
    double *lpt;                        // [B]
    float *tape_s_next;                 // [d_s][B] slot of s_{t+1}, or null
    float *states_out_next;             // [B][d_s] or null
    const float *goals_t, *goals_next;  // [B][d_g]; goals_next null at the last step
    float *jdst;                        // tape slot [M][D][B] of step t, or null
};

// p[0] + p[stride] + ... (n terms, added in that order); the loads go out eight at a time so that
// their latencies overlap (one round trip for up to eight work-unit groups)
__device__ __forceinline__ double sum_groups(const double *__restrict__ p, int n, size_t stride)
{
    double s = 0.0;
    for (int c0 = 0; c0 < n; c0 += 8) {
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = (c0 + u < n) ? p[(size_t)(c0 + u) * stride] : 0.0;
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    return s;
}

// The first eight terms of such a sum, requested only (pinned where they are written, see load16_pinned, so
// that the compiler does not sink them below the weight loads that follow); the caller adds them up later.
__device__ __forceinline__ void request_groups(const double *__restrict__ p, int n, size_t stride, unsigned long long (&v)[8])
{
#pragma unroll
    for (int u = 0; u < 8; ++u)
        v[u] = (u < n) ? __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p + (size_t)u * stride),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT)
                       : 0ull;
}

__global__ __launch_bounds__(PW * 64) void step_tail_kernel(tail_args r, policy_args a)
{
    __shared__ float4 act4[(BAGEL_MAX_HIDDEN / 4) * PL];
    __shared__ float4 red4[PW * 4 * 64];
    __shared__ __align__(16) float biasS[3][BAGEL_MAX_HIDDEN];
    __shared__ double fS[16][PL], sS[8][PL];             // fS rows: u sums, then (from row M) feature sums
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b0 = blockIdx.x * PL;
    const int bl = tid & (PL - 1), row = tid >> 5;      // 16 rows x 32 trajectories
    const bool liveq = b0 + bl < a.B;
    const int bq = liveq ? b0 + bl : a.B - 1;
    const int B = a.B, ds = a.ds;
    const int d_in = a.width[0];                        // d_s + d_g <= 16: one policy input row per thread row

    // Everything the end of the step reads from global memory is requested here, before anything waits
    // for a value: the kernel is a chain of latencies, and they overlap only if they start together.
    // The order matters as well: a wave consumes its loads in the order it issued them, so the value sums
    // (needed first) go out before the 264 KB of weights (needed by the second layer); issued after them
    // they were not usable before the last weight had arrived (4.4 us into the kernel instead of 1.5).
    double x_in = 0.0, lp_in = 0.0;
    float g_in = 0.0f, gt_in[8];
    if (row < ds) x_in = r.x_cur[(size_t)row * B + bq];
    else if (row < d_in && r.goals_next) g_in = r.goals_next[(size_t)bq * r.dg + (row - ds)];
    if (r.add_cost && row == 0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) gt_in[j] = j < r.dg ? r.goals_t[(size_t)bq * r.dg + j] : 0.0f;
        lp_in = r.lpt[bq];
    }

    // ---- value sums -> LDS: thread row m adds the kernel-row sums of output m, row M + m its feature
    // sums.  (direct: part holds f and J_f themselves, one (output, component) pair per thread row and
    // pass; J_f goes to the tape from here.)
    const size_t stride = (size_t)(1 + r.D) * B;
    unsigned long long vreq[8] = {};
    const double *vsrc = nullptr;
    int vn = 0;
    if (r.direct) {
        for (int qi = row; qi < r.M * r.ncomp; qi += 16) {
            const int m = qi / r.ncomp, comp = qi - m * r.ncomp;
            const double val = r.part[(size_t)m * stride + (size_t)comp * B + bq];
            if (comp == 0) fS[m][bl] = val;
            else if (liveq) r.jdst[(size_t)(m * r.D + comp - 1) * B + bq] = (float)val;
        }
    } else if (row < r.M) {
        vsrc = r.part + (size_t)(row * r.ngk) * stride + bq;
        vn = r.ngk;
    } else if (row < 2 * r.M) {
        vsrc = r.part + (size_t)(r.M * r.ngk + (row - r.M) * r.ngl) * stride + bq;
        vn = r.ngl;
    }
    if (vn > 0) request_groups(vsrc, vn, stride, vreq);
    FORWARD_WEIGHTS_DECL;
    if (r.do_policy) load_forward_weights(a, wave, lane, w_first, w_last, w_wide, p_first, p_last, p_wide, bias_r);
    if (vn > 0) {
        double vsum = 0.0;
#pragma unroll
        for (int u = 0; u < 8; ++u) vsum += __longlong_as_double((long long)vreq[u]);      // absent terms are +0.0
        if (vn > 8) vsum += sum_groups(vsrc + 8 * stride, vn - 8, stride);
        fS[row][bl] = vsum;
    }
    __syncthreads();

    // ---- s_{t+1}, tapes, and the policy input [s_{t+1} ; g_{t+1}] (rows up to 32 zero) in act4
    float *act1 = reinterpret_cast<float *>(act4);
    {
        float hin = 0.0f;
        if (row < ds) {
            const double f = r.direct ? fS[row][bl] : r.amp[row] * fS[r.M + row][bl] + fS[row][bl];
            const double sn = x_in + f;
            sS[row][bl] = sn;
            hin = (float)sn;
            if (liveq) {
                r.x_next[(size_t)row * B + bq] = sn;
                if (r.tape_s_next) r.tape_s_next[(size_t)row * B + bq] = hin;
                if (r.states_out_next) r.states_out_next[(size_t)bq * ds + row] = hin;
            }
        } else if (row < d_in) {
            hin = g_in;
        }
        if (r.do_policy) {
            act1[((row >> 2) * PL + bl) * 4 + (row & 3)] = hin;
            act1[(((row + 16) >> 2) * PL + bl) * 4 + (row & 3)] = 0.0f;
            if (liveq && row < d_in) a.h[0][(size_t)row * B + bq] = hin;
        }
    }
    if (r.do_policy) stash_biases(a, bias_r, biasS);
    __syncthreads();
    if (r.add_cost && row == 0 && liveq) {
        double e = 0.0;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (j < r.dg) {
                const double dlt = sS[r.tracked[j]][bl] - (double)gt_in[j];
                e += (double)r.q[j] * dlt * dlt;
            }
        if (r.cost_kind == 1) {
            const double sr2 = (double)r.sigma_r * (double)r.sigma_r;
            e = -exp(-e / (2.0 * sr2));
        }
        r.lpt[bq] = lp_in + e;
    }
    if (r.do_policy) policy_layers(a, w_first, w_last, w_wide, p_first, p_last, p_wide, wave, lane, b0, act4, red4, biasS);
}

// ---- backward sweep ------------------------------------------------------------------------
// Reverse-mode pass of Algorithm 1 over the steps t_hi-1, ..., t_lo of every trajectory in ONE
// launch.  Trajectories do not interact in the sweep, so a workgroup keeps its 32 trajectories for
// the whole range and walks the tape backwards on its own; the adjoint of the state (lam) lives in
// LDS in float64.  For step k = t-1 (tape slot k - t_lo), with lam = lam_t = dL/ds_t:
//   u      = J_f(x_k)^T lam                         (J_f from the tape, [M][D])
//   us     = u[:d_s];  delta_out = u[d_s:] * d a / d z_out   -> tape_d[last], input of the policy backward
//   policy backward through W^T (matrix cores): tape_d[l-1] for the weight-gradient GEMM, and the
//   adjoint dh0 of the policy input, whose first d_s rows are (d a_k / d s_k)^T u_a
//   lam_{t-1} = lam + us + dh0[:d_s] + [t-1 >= 1] (1/B) d cost / d s (s_{t-1}, g_{t-2})
// lam_{t_hi} is the cost gradient at s_H when t_hi == H and is read from `lam` otherwise (the sweep
// of a checkpointed rollout is split into segments); lam_{t_lo} is written back to `lam`, and to
// grad_s0 when t_lo == 0.
struct sweep_args {
    int B, nl, ds, da, dg, D, M, H;
    int t_hi, t_lo;
    int width[4];
    int wp_off[3], kp[3];
    float act_bound;
    int cost_kind;
    float sigma_r;
    int tracked[8];
    float q[8];
    const float *Wp;          // packed backward weights
    const float *tape_h[3];   // slot 0 of each tape
    float *tape_d[3];
    const float *tape_a, *tape_J, *tape_s;
    const float *goals;       // [H][B][d_g]
    double *lam;              // [d_s][B]
    float *grad_s0;           // [B][d_s] or null
};

// 4-byte read that the optimiser keeps where it is written (see load16_pinned).  Used for the tape
// values a later phase needs, requested a phase early so that they arrive under the matrix work.
__device__ __forceinline__ float load_pinned(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}

__device__ __forceinline__ const float *at_byte(const float *base, unsigned byte_off)
{
    return reinterpret_cast<const float *>(reinterpret_cast<const char *>(base) + byte_off);
}

// What thread (row, trajectory) reads from the tape for one step of the sweep: row d < D owns
// component d of u = J^T lam.
struct sweep_tape {
    float J[8];           // J[m][row]
    float th;             // rows d_s .. D-1: tanh output of the bounded action row - d_s
};
struct sweep_cost {
    float sv[8], gv[8];   // tracked states of s_{t-1} and the goals they are compared with
};

// step k = t-1 (tape slot k - t_lo) and the cost data of state t-1.  Addresses: wave-uniform slot and row
// bases plus one 32-bit lane offset (see at_byte); spelled out per access as 64-bit vector arithmetic they
// cost more instructions than the loads themselves.
__device__ __forceinline__ void sweep_tape_load(const sweep_args &a, int t, int row, int bq, sweep_tape &r)
{
    const size_t slot = (size_t)(t - 1 - a.t_lo);
    const unsigned B = (unsigned)a.B, ubq = (unsigned)bq;
    // All loads are issued without conditions (indices past M, d_g are clamped to the last one, rows past
    // D to the last row: duplicates that nothing reads): with a branch per load the compiler must assume at
    // every join that an earlier load may still be writing the registers it is about to reuse, and makes
    // each load wait for the one before.
    {
        const int rowc = row < a.D ? row : a.D - 1;
        const float *Jt = a.tape_J + slot * a.M * a.D * a.B;
        const unsigned off = ((unsigned)rowc * B + ubq) * 4u;
#pragma unroll
        for (int m = 0; m < 8; ++m) r.J[m] = load_pinned(at_byte(Jt + (size_t)(m < a.M ? m : a.M - 1) * a.D * a.B, off));
        const int ra = rowc >= a.ds ? rowc - a.ds : 0;
        r.th = load_pinned(at_byte(a.tape_a + slot * a.da * a.B, ((unsigned)ra * B + ubq) * 4u));
    }
}

// The cost data of state t-1, which the end of step t needs: requested at the start of that same step (a
// whole step ahead of their use; a second register set for them would not pay).
__device__ __forceinline__ void sweep_cost_load(const sweep_args &a, int t, int bq, sweep_cost &r)
{
    const unsigned ubq = (unsigned)bq;
    const int tc = t - 1 >= 1 ? t : 2;                   // they exist for t-1 >= 1; otherwise any valid slot
    const float *st = a.tape_s + (size_t)(tc - 1) * a.ds * a.B;
    const float *gt = a.goals + (size_t)(tc - 2) * a.B * a.dg;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int jc = j < a.dg ? j : a.dg - 1;
        r.sv[j] = load_pinned(at_byte(st + (size_t)a.tracked[jc] * a.B, ubq * 4u));
        r.gv[j] = load_pinned(at_byte(gt + jc, ubq * (unsigned)a.dg * 4u));
    }
}

// lam + (1/B) d cost / d s_i, the cost of tracked states sv against goals gv
__device__ __forceinline__ double add_cost_gradient(const sweep_args &a, double lam, int i, const float *sv,
                                                    const float *gv)
{
    double r[8], e = 0.0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        r[j] = 0.0;
        if (j < a.dg) {
            r[j] = (double)sv[j] - (double)gv[j];
            e += (double)a.q[j] * r[j] * r[j];
        }
    }
    double factor = 2.0;
    if (a.cost_kind == 1) {
        const double sr2 = (double)a.sigma_r * (double)a.sigma_r;
        factor = exp(-e / (2.0 * sr2)) / sr2;
    }
    factor /= (double)a.B;
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (j < a.dg && a.tracked[j] == i) lam += factor * (double)a.q[j] * r[j];
    return lam;
}

// tanh outputs h_l of the units a wave owns (the rows of its output tile), for the tanh derivative.
// hl: the layer's tape slot (wave-uniform); lane_off: byte offset of (row 4 hf, the lane's trajectory).
// The scalar row base is clamped to the layer's last row; with the lane's four rows on top a lane whose
// unit does not exist reads up to four rows further (the next slot, or the slack behind the last one) and
// does not use what it gets.
__device__ __forceinline__ void load_tanh_outputs(const float *hl, int ni, int B, unsigned lane_off, const wave_plan &p,
                                                  float *hv)
{
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int iu = min(p.rt * 32 + 8 * g + e, ni - 1);
            hv[4 * g + e] = load_pinned(at_byte(hl + (size_t)iu * B, lane_off));
        }
}

__global__ __launch_bounds__(PW * 64) void backward_sweep_kernel(sweep_args a)
{
    __shared__ float4 act4[(BAGEL_MAX_HIDDEN / 4) * PL];
    __shared__ float4 red4[PW * 4 * 64];
    __shared__ double lamS[8][PL], usS[8][PL];
    __shared__ float dh0S[16][PL];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31, hf = lane >> 5;
    const int b0 = blockIdx.x * PL;
    const int b = b0 + c;
    const bool live = b < a.B;
    const int bc = live ? b : a.B - 1;            // clamped trajectory of the MFMA lanes
    const unsigned lane_off = ((unsigned)(4 * hf) * (unsigned)a.B + (unsigned)bc) * 4u;   // (row 4 hf, trajectory)
    const int last = a.nl - 1;
    // the lane-per-(row, trajectory) phases see the workgroup as 16 rows x 32 trajectories
    const int bl = tid & (PL - 1), row = tid >> 5;
    const bool liveq = b0 + bl < a.B;
    const int bq = liveq ? b0 + bl : a.B - 1;
    // the wave's share of the top layer (input width[last], contraction over the d_a outputs)
    const wave_plan p_top = plan_layer(a.width[last], a.kp[last], wave);
    const bool top_owner = last > 0 && p_top.active && p_top.ks == 0;

    if (row < a.ds) {
        double v = 0.0;
        if (a.t_hi == a.H) {
            float sv[8], gv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (j < a.dg) {
                    sv[j] = a.tape_s[((size_t)a.H * a.ds + a.tracked[j]) * a.B + bq];
                    gv[j] = a.goals[((size_t)(a.H - 1) * a.B + bq) * a.dg + j];
                }
            v = add_cost_gradient(a, 0.0, row, sv, gv);
        } else {
            v = a.lam[(size_t)row * a.B + bq];
        }
        lamS[row][bl] = v;
    }
    // The wave's share of the two narrow transposed weight matrices stays in registers for the whole
    // sweep (top layer: one group, its contraction runs over the d_a <= 8 outputs); the wide middle
    // layer is streamed from L2 every step.
    const wave_plan p_first = plan_layer(a.width[0], a.kp[0], wave);
    float4 w_first[4];
    load_wave_weights<1>(w_first, a.Wp + a.wp_off[0], a.kp[0], p_first, lane);
    const float4 w_top = reinterpret_cast<const float4 *>(a.Wp + a.wp_off[last])[(size_t)p_top.rt * (a.kp[last] >> 3) * 64 + lane];
    const wave_plan p_mid = last == 2 ? plan_layer(a.width[1], a.kp[1], wave) : p_first;
    sweep_tape cur = {}, nxt = {};
    sweep_cost cost = {};
    float hv_top[16] = {}, hv_top_next[16] = {};
    sweep_tape_load(a, a.t_hi, row, bq, cur);
    if (top_owner)
        load_tanh_outputs(a.tape_h[last] + (size_t)(a.t_hi - 1 - a.t_lo) * a.width[last] * a.B, a.width[last], a.B,
                          lane_off, p_top, hv_top);
    __syncthreads();

    for (int t = a.t_hi; t > a.t_lo; --t) {
        const size_t slot = (size_t)(t - 1 - a.t_lo);
        // ---- u = J^T lam, one component per row: the state part goes to usS, the action part times
        //      d a / d z_out is the input of the policy backward (rows d_a .. 31 of it are zero: one MFMA
        //      batch consumes 32 rows)
        float *act1 = reinterpret_cast<float *>(act4);
        if (tid < 6 * PL) act4[(2 + row) * PL + bl] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (row < a.D) {
            double acc = 0.0;
#pragma unroll
            for (int m = 0; m < 8; ++m)
                if (m < a.M) acc += (double)cur.J[m] * lamS[m][bl];
            if (row < a.ds) {
                usS[row][bl] = acc;
            } else {
                const int o = row - a.ds;
                if (a.act_bound > 0.0f) {
                    const double th = (double)cur.th;
                    acc *= (double)a.act_bound * (1.0 - th * th);
                }
                const float dv = (float)acc;
                if (liveq) a.tape_d[last][(slot * a.da + o) * a.B + bq] = dv;
                act1[((o >> 2) * PL + bl) * 4 + (o & 3)] = dv;
            }
        } else if (row - a.ds < 8) {
            const int o = row - a.ds;
            act1[((o >> 2) * PL + bl) * 4 + (o & 3)] = 0.0f;
        }
        __syncthreads();
        // the cost data this step ends with, and the tape of the next step of the sweep, are requested now
        // and arrive under the matrix work
        sweep_cost_load(a, t, bq, cost);
        if (t - 1 > a.t_lo) {
            sweep_tape_load(a, t - 1, row, bq, nxt);
            if (top_owner)
                load_tanh_outputs(a.tape_h[last] + (slot - 1) * a.width[last] * a.B, a.width[last], a.B, lane_off, p_top,
                                  hv_top_next);
        }

        // ---- policy backward: delta_{l-1} = (W_l^T delta_l) * (1 - h_l^2).  The layers are written out one
        // after the other (top, middle if there are three, first) instead of a loop over l: a loop carries
        // the accumulator from one trip to the next through register copies, and with loads in flight the
        // compiler guards every such copy with a wait for all of them, the next step's tape values included.
        auto backward_layer = [&](auto kind_tag, int l, const wave_plan &p) {
            constexpr int KIND = decltype(kind_tag)::value;          // 2: top, 1: middle, 0: first
            const int ni = a.width[l];
            const bool owner = p.active && p.ks == 0;
            float hv[16];
            if (KIND == 1 && owner) load_tanh_outputs(a.tape_h[l] + slot * ni * a.B, ni, a.B, lane_off, p, hv);
            f16v acc;
            if (p.active) {
                if (KIND == 2) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
                    acc = mfma_group(acc, w_top, act4[hf * PL + c]);
                } else if (KIND == 0) {
                    acc = contract_batches<1>(w_first, p, lane, act4);
                } else {
                    acc = tile_contract(a.Wp + a.wp_off[l], a.kp[l], p, lane, act4);
                }
            }
            if (KIND == 0 && p.ksplit > 1) {
                // the adjoint of the policy input: one row tile (at most 16 rows are used), the contraction
                // split over up to eight waves.  Every slice goes to LDS and 128 threads add them up, four
                // rows of one trajectory each, in slice order (one wave adding seven slices to its own took
                // 1.5 us of a 20 us step).
                if (p.active) {
#pragma unroll
                    for (int g = 0; g < 2; ++g)
                        red4[(wave * 4 + g) * 64 + lane] = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
                }
                __syncthreads();
                if (tid < 128) {
                    const int g = tid >> 6, ln = tid & 63;
                    float4 t4 = red4[(0 * 4 + g) * 64 + ln];
                    for (int sl = 1; sl < p.ksplit; ++sl) {
                        const float4 u4 = red4[(sl * 4 + g) * 64 + ln];
                        t4.x += u4.x; t4.y += u4.y; t4.z += u4.z; t4.w += u4.w;
                    }
                    const int ib = 8 * g + 4 * (ln >> 5);
                    const float o4[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (ib + e < ni) dh0S[ib + e][ln & 31] = o4[e];
                }
                __syncthreads();
                return;
            }
            combine_slices(acc, p, wave, lane, red4);
            if (owner) {
                float *drow = KIND > 0 ? a.tape_d[l - 1] + (slot * ni + p.rt * 32) * a.B : nullptr;    // wave-uniform
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int ib = p.rt * 32 + 8 * g + 4 * hf;
                    float out[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int i = ib + e;
                        float dv = 0.0f;
                        if (i < ni) {
                            dv = acc[4 * g + e];
                            if (KIND > 0) {
                                const float h = KIND == 2 ? hv_top[4 * g + e] : hv[4 * g + e];
                                dv *= (1.0f - h * h);
                                if (live) *at_byte(drow + (size_t)(8 * g + e) * a.B, lane_off) = dv;
                            } else if (i < 16) {
                                dh0S[i][c] = dv;
                            }
                        }
                        out[e] = dv;
                    }
                    if (KIND > 0) act4[(ib >> 2) * PL + c] = make_float4(out[0], out[1], out[2], out[3]);
                }
            }
            __syncthreads();
        };
        if (last > 0) backward_layer(std::integral_constant<int, 2>{}, last, p_top);
        if (last == 2) backward_layer(std::integral_constant<int, 1>{}, 1, p_mid);
        backward_layer(std::integral_constant<int, 0>{}, 0, p_first);

        // ---- lam_{t-1}
        if (row < a.ds) {
            double v = lamS[row][bl] + usS[row][bl] + (double)dh0S[row][bl];
            if (t - 1 >= 1) v = add_cost_gradient(a, v, row, cost.sv, cost.gv);
            lamS[row][bl] = v;
        }
        cur = nxt;
#pragma unroll
        for (int r = 0; r < 16; ++r) hv_top[r] = hv_top_next[r];
        __syncthreads();
    }

    if (row < a.ds && liveq) {
        const double v = lamS[row][bl];
        a.lam[(size_t)row * a.B + bq] = v;
        if (a.t_lo == 0 && a.grad_s0) a.grad_s0[(size_t)bq * a.ds + row] = (float)v;
    }
}

// theta -> packed, zero-padded forward (rows = outputs, K = inputs) and backward (rows = inputs,
// K = outputs) matrices in the fragment order tile_contract and load_wave_weights read
__device__ __forceinline__ void unpack_index(int idx, int kp, int &row, int &k)
{
    const int e = idx & 3, lane = (idx >> 2) & 63, blk = idx >> 8;     // blk = rt * (kp/8) + k8
    const int k8 = blk % (kp >> 3), rt = blk / (kp >> 3);
    row = rt * 32 + (lane & 31);
    k = k8 * 8 + 4 * (lane >> 5) + e;
}

__global__ void pack_theta_kernel(const float *__restrict__ theta, float *__restrict__ Wf, float *__restrict__ Wb,
                                  int no, int ni, int w_off, int f_off, int f_rp, int f_kp, int b_off, int b_rp,
                                  int b_kp)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < f_rp * f_kp) {
        int j, k;
        unpack_index(idx, f_kp, j, k);
        Wf[f_off + idx] = (j < no && k < ni) ? theta[w_off + j * ni + k] : 0.0f;
    }
    if (idx < b_rp * b_kp) {
        int i, o;
        unpack_index(idx, b_kp, i, o);
        Wb[b_off + idx] = (i < ni && o < no) ? theta[w_off + o * ni + i] : 0.0f;
    }
}

// ---- weight gradient GEMM ------------------------------------------------------------------
// C[o][i] = sum_kk Dl[o][kk] * Hl[i][kk], kk = (slot, b); db[o] = sum_kk Dl[o][kk].
// Wave (wr, wc) of a wrows x wcols wave grid (at most 4x4, sized to the layer so that no wave idles)
// owns rows [64 wr, +64) x columns [64 wc, +64) as 2x2 MFMA tiles.
template <bool FAST>
__global__ __launch_bounds__(1024) void weight_grad_kernel(const float *__restrict__ Dl, const float *__restrict__ Hl,
                                                           float *__restrict__ gsplit, int no, int ni, int B,
                                                           int n_slots, int chunks_per_slot, int chunks_per_split,
                                                           int w_off, int b_off, int P, int wcols)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wr = wave / wcols, wc = wave - wr * wcols;   // the workgroup has wrows x wcols waves
    const int cl = lane & 31, hf = lane >> 5;
    const int o_base = blockIdx.y * 256 + wr * 64, i_base = blockIdx.z * 256 + wc * 64;
    if (o_base >= no || i_base >= ni) return;   // whole wave has nothing to do (no barriers in this kernel)
    const bool fa_on[2] = {true, o_base + 32 < no};
    const bool fb_on[2] = {true, i_base + 32 < ni};
    const int total_chunks = n_slots * chunks_per_slot;
    const int c_begin = blockIdx.x * chunks_per_split;
    const int c_end = min(total_chunks, c_begin + chunks_per_split);

    f16v acc[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.0f;
    float bsum[2] = {0.0f, 0.0f};
    const int orow[2] = {o_base + cl, o_base + 32 + cl};
    const int irow[2] = {i_base + cl, i_base + 32 + cl};
    // rows past the end are clamped: they feed accumulator rows / columns that are never stored
    const int oc[2] = {min(orow[0], no - 1), min(orow[1], no - 1)};
    const int ic[2] = {min(irow[0], ni - 1), min(irow[1], ni - 1)};

    auto mfma_chunk = [&](const float4 *a4, const float4 *b4) {
#pragma unroll
        for (int f = 0; f < 2; ++f) bsum[f] += (a4[f].x + a4[f].y) + (a4[f].z + a4[f].w);
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            if (!fa_on[x]) continue;
#pragma unroll
            for (int y = 0; y < 2; ++y) {
                if (!fb_on[y]) continue;
                acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[x].x, b4[y].x, acc[x][y], 0, 0, 0);
                acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[x].y, b4[y].y, acc[x][y], 0, 0, 0);
                acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[x].z, b4[y].z, acc[x][y], 0, 0, 0);
                acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[x].w, b4[y].w, acc[x][y], 0, 0, 0);
            }
        }
    };

    if (FAST) {
        // B % 8 == 0: every chunk is full and 16-byte aligned; loads are unconditional and the operands
        // of chunk c+1 are requested before the MFMAs of chunk c issue
        auto load_chunk = [&](int c, float4 *a4, float4 *b4) {
            const int slot = c / chunks_per_slot;
            const int bb = (c - slot * chunks_per_slot) * 8 + 4 * hf;
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                a4[f] = *reinterpret_cast<const float4 *>(Dl + ((size_t)slot * no + oc[f]) * B + bb);
                b4[f] = *reinterpret_cast<const float4 *>(Hl + ((size_t)slot * ni + ic[f]) * B + bb);
            }
        };
        float4 a4[2], b4[2], an[2], bn[2];
        if (c_begin < c_end) load_chunk(c_begin, a4, b4);
        for (int c = c_begin; c < c_end; ++c) {
            load_chunk(c + 1 < c_end ? c + 1 : c, an, bn);
            mfma_chunk(a4, b4);
#pragma unroll
            for (int f = 0; f < 2; ++f) { a4[f] = an[f]; b4[f] = bn[f]; }
        }
    } else {
        for (int c = c_begin; c < c_end; ++c) {
            const int slot = c / chunks_per_slot;
            const int bb = (c - slot * chunks_per_slot) * 8 + 4 * hf;
            float4 a4[2], b4[2];
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                const float *ar = Dl + ((size_t)slot * no + oc[f]) * B;
                const float *br = Hl + ((size_t)slot * ni + ic[f]) * B;
                float ta[4], tb[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool ok = bb + e < B;
                    ta[e] = ok ? ar[bb + e] : 0.0f;
                    tb[e] = ok ? br[bb + e] : 0.0f;
                }
                a4[f] = make_float4(ta[0], ta[1], ta[2], ta[3]);
                b4[f] = make_float4(tb[0], tb[1], tb[2], tb[3]);
            }
            mfma_chunk(a4, b4);
        }
    }
    float *g = gsplit + (size_t)blockIdx.x * P;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int o = o_base + x * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
                const int i = i_base + y * 32 + cl;
                if (o < no && i < ni) g[w_off + (size_t)o * ni + i] = acc[x][y][r];
            }
    if (blockIdx.z == 0 && wc == 0) {
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            const float tot = bsum[f] + __shfl_xor(bsum[f], 32);
            if (hf == 0 && orow[f] < no) g[b_off + orow[f]] = tot;
        }
    }
}

// The same GEMM with both operands staged through LDS (B a multiple of 32).  The direct kernel above
// has every lane fetch 16 bytes of a row of its own per chunk: a wave instruction touches 32 cache
// lines for 1 KB, every line is asked for four times, and the kernel is held by the rate at which
// the vector cache can look lines up (3.4 TB/s on a skinny layer), or by the L2-to-CU bandwidth on a
// wide one.  Here the waves of a workgroup bring one tile of 32 contraction indices (32 trajectories
// of one tape slot) for all rows of both operands into LDS with loads that write LDS directly (no
// staging registers: on the wide layer the accumulators, the operand fragments of two contraction
// steps and the addresses are all that a wave's 128 registers hold).  Such a load puts lane i's 16
// bytes at byte 16 i of the wave's 1 KB destination, so a wave instruction carries 8 whole rows of
// 128 bytes and the rows sit unpadded; the lane that fills the 16-byte column q of row r fetches
// column q ^ (r & 7) of that row instead, which spreads the fragment reads of 8 consecutive rows
// over all banks.  NST stages: the loads of tiles k+1 .. k+NST-1 are in flight while the MFMAs of
// tile k run; one barrier per tile.
//   WA x WB waves, each TA x TB MFMA tiles of 32 x 32: the workgroup covers 32 WA TA rows (outputs)
//   and 32 WB TB columns (inputs); rows and columns past the layer's are clamped duplicates whose
//   accumulators are never stored.  Instances: 4 x 4 waves of 2 x 2 tiles for a wide layer (both
//   sides in (128, 256]); 8 x 1 and 1 x 8 waves of one tile for a skinny one (one side <= 32).
constexpr int WG_KC = 32;              // contraction indices per tile

// One wave instruction: lane i's 16 bytes at g go to LDS byte address lds_addr + 16 i (lds_addr is
// wave-uniform).  Written as assembly so that the loads of the next tile stay in flight under the
// fragment reads of the current one: the compiler orders every LDS read after all outstanding loads
// of this kind, whichever part of LDS they fill.  No register is written, so nothing the compiler
// allocates depends on the load's completion; the caller waits (vmcnt) before the barrier that
// publishes the tile.  M0 carries the LDS address; the kernel that calls this uses M0 for nothing else.
__device__ __forceinline__ void load_16_bytes_per_lane_to_lds(const float *g, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(lds_addr) : "memory");
}

// s_waitcnt with only the vector-memory counter set (expcnt and lgkmcnt left at their maxima)
template <int N>
__device__ __forceinline__ void wait_vector_loads_at_most()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

template <int WA, int WB, int TA, int TB, int NST>
struct wg_tiling {
    static constexpr int NW = WA * WB;                       // waves
    static constexpr int RA = 32 * WA * TA, RB = 32 * WB * TB;   // rows of the two operands the MFMAs read
    // rows brought into LDS: rounded up so that every wave issues the same number of loads per tile
    static constexpr int LA = (RA + 8 * NW - 1) / (8 * NW) * (8 * NW), LB = (RB + 8 * NW - 1) / (8 * NW) * (8 * NW);
    static constexpr int NA = LA / (8 * NW), NB = LB / (8 * NW);   // loads per wave and tile
    static constexpr int STAGE = (LA + LB) * WG_KC;          // floats per stage: A rows, then B rows
    static constexpr size_t LDS_BYTES = (size_t)NST * STAGE * sizeof(float);
};

template <int WA, int WB, int TA, int TB, int NST>
__global__ __launch_bounds__(64 * WA * WB) void weight_grad_tiled_kernel(const float *__restrict__ Dl,
                                                                         const float *__restrict__ Hl,
                                                                         float *__restrict__ gsplit, int no, int ni, int B,
                                                                         int n_slots, int tiles_per_split, int w_off,
                                                                         int b_off, int P)
{
    using T = wg_tiling<WA, WB, TA, TB, NST>;
    extern __shared__ float lds[];     // [NST stages][A: LA x WG_KC | B: LB x WG_KC]
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) float *)lds;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave / WB, wc = wave - wr * WB;
    const int cl = lane & 31, hf = lane >> 5;
    const int tiles_per_slot = B / WG_KC;
    const int total = n_slots * tiles_per_slot;
    const int t_begin = blockIdx.x * tiles_per_split;
    const int t_end = min(total, t_begin + tiles_per_split);

    // global -> LDS: load j of a wave brings rows [8 (j NW + wave), +8) of an operand
    const int lr = lane >> 3;                                   // row within the instruction's 8
    const int lq = (lane & 7) ^ lr;                             // 16-byte column this lane fetches
    size_t offa[T::NA], offb[T::NB];                            // element offsets within a slot, column included
#pragma unroll
    for (int j = 0; j < T::NA; ++j) offa[j] = (size_t)min(8 * (j * T::NW + wave) + lr, no - 1) * B + 4 * lq;
#pragma unroll
    for (int j = 0; j < T::NB; ++j) offb[j] = (size_t)min(8 * (j * T::NW + wave) + lr, ni - 1) * B + 4 * lq;
    // position of the next tile to load: first element of its 32 trajectories in row 0 of its slot
    int ld_tb = t_begin % tiles_per_slot;
    const float *ga = Dl + (size_t)(t_begin / tiles_per_slot) * no * B + ld_tb * WG_KC;
    const float *gb = Hl + (size_t)(t_begin / tiles_per_slot) * ni * B + ld_tb * WG_KC;
    auto load_next_tile = [&](int stage) {
        const unsigned la = lds_base + (unsigned)(stage * T::STAGE + 8 * wave * WG_KC) * 4u, lb = la + T::LA * WG_KC * 4;
#pragma unroll
        for (int j = 0; j < T::NA; ++j) load_16_bytes_per_lane_to_lds(ga + offa[j], la + 8 * j * T::NW * WG_KC * 4);
#pragma unroll
        for (int j = 0; j < T::NB; ++j) load_16_bytes_per_lane_to_lds(gb + offb[j], lb + 8 * j * T::NW * WG_KC * 4);
        if (++ld_tb == tiles_per_slot) {
            ld_tb = 0;
            ga += (size_t)no * B - (size_t)(tiles_per_slot - 1) * WG_KC;
            gb += (size_t)ni * B - (size_t)(tiles_per_slot - 1) * WG_KC;
        } else {
            ga += WG_KC;
            gb += WG_KC;
        }
    };

    f16v acc[TA][TB];
#pragma unroll
    for (int x = 0; x < TA; ++x)
#pragma unroll
        for (int y = 0; y < TB; ++y)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.0f;
    float bsum[TA];
#pragma unroll
    for (int x = 0; x < TA; ++x) bsum[x] = 0.0f;

#pragma unroll
    for (int k = 0; k < NST - 1; ++k)
        if (t_begin + k < t_end) load_next_tile(k);
    // the first tile is in LDS once every wave's share of it is; later tiles may still be in flight
    if (t_begin + NST - 1 <= t_end) wait_vector_loads_at_most<(NST - 2) * (T::NA + T::NB)>();
    else wait_vector_loads_at_most<0>();
    __syncthreads();
    // fragment reads: row 32 (wr TA + f) + cl (its low three bits are cl's), 16-byte column (2 k8 + hf) ^ (cl & 7)
    const int sw = cl & 7;
    const float *Ar = lds + (32 * TA * wr + cl) * WG_KC, *Br = lds + T::LA * WG_KC + (32 * TB * wc + cl) * WG_KC;
    int stage = 0, ld_stage = NST - 1;
    for (int t = t_begin; t < t_end; ++t) {
        const bool more = t + NST - 1 < t_end;
        if (more) load_next_tile(ld_stage);     // into the stage that tile t-1 was read from
        const float *As = Ar + stage * T::STAGE, *Bs = Br + stage * T::STAGE;
#pragma unroll
        for (int k8 = 0; k8 < WG_KC / 8; ++k8) {
            const int col = 4 * ((2 * k8 + hf) ^ sw);
            float4 a4[TA], b4[TB];
#pragma unroll
            for (int f = 0; f < TA; ++f) a4[f] = *reinterpret_cast<const float4 *>(As + 32 * f * WG_KC + col);
#pragma unroll
            for (int f = 0; f < TB; ++f) b4[f] = *reinterpret_cast<const float4 *>(Bs + 32 * f * WG_KC + col);
#pragma unroll
            for (int f = 0; f < TA; ++f) bsum[f] += (a4[f].x + a4[f].y) + (a4[f].z + a4[f].w);
#pragma unroll
            for (int x = 0; x < TA; ++x)
#pragma unroll
                for (int y = 0; y < TB; ++y) {
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[x].x, b4[y].x, acc[x][y], 0, 0, 0);
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[x].y, b4[y].y, acc[x][y], 0, 0, 0);
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[x].z, b4[y].z, acc[x][y], 0, 0, 0);
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[x].w, b4[y].w, acc[x][y], 0, 0, 0);
                }
        }
        // tile t+1 has landed (loads complete in order; those of later tiles may stay in flight)
        if (more) wait_vector_loads_at_most<(NST - 2) * (T::NA + T::NB)>();
        else wait_vector_loads_at_most<0>();
        __syncthreads();
        stage = stage + 1 == NST ? 0 : stage + 1;
        ld_stage = ld_stage + 1 == NST ? 0 : ld_stage + 1;
    }

    float *g = gsplit + (size_t)blockIdx.x * P;
    const int o_base = 32 * TA * wr, i_base = 32 * TB * wc;
#pragma unroll
    for (int x = 0; x < TA; ++x)
#pragma unroll
        for (int y = 0; y < TB; ++y)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int o = o_base + x * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
                const int i = i_base + y * 32 + cl;
                if (o < no && i < ni) g[w_off + (size_t)o * ni + i] = acc[x][y][r];
            }
    if (wc == 0) {
#pragma unroll
        for (int f = 0; f < TA; ++f) {
            const float tot = bsum[f] + __shfl_xor(bsum[f], 32);
            const int o = o_base + 32 * f + cl;
            if (hf == 0 && o < no) g[b_off + o] = tot;
        }
    }
}

// gacc[p] (+)= sum_z gsplit[z][p]; optionally emit grad_theta = (float) gacc.  64 parameters per workgroup;
// wave q adds the q-th quarter of the splits in z order, the four quarters are added in order.
__global__ __launch_bounds__(256) void grad_reduce_kernel(const float *__restrict__ gsplit, double *__restrict__ gacc, int P,
                                                          int ksplit, bool accumulate, float *__restrict__ grad_theta)
{
    __shared__ double sh[4][64];
    const int lane = threadIdx.x & 63, quarter = threadIdx.x >> 6;
    const int p = blockIdx.x * 64 + lane;
    const int per = (ksplit + 3) / 4;
    const int z0 = quarter * per, z1 = min(ksplit, z0 + per);
    double s = 0.0;
    if (p < P) {
#pragma unroll 8
        for (int z = z0; z < z1; ++z) s += (double)gsplit[(size_t)z * P + p];
    }
    sh[quarter][lane] = s;
    __syncthreads();
    if (quarter == 0 && p < P) {
        const double tot = (accumulate ? gacc[p] : 0.0) + (((sh[0][lane] + sh[1][lane]) + sh[2][lane]) + sh[3][lane]);
        gacc[p] = tot;
        if (grad_theta) grad_theta[p] = (float)tot;
    }
}

// Adam update (Kingma & Ba, Algorithm 1) of theta, m, v in place; corr1 = 1 - beta1^step, corr2 = 1 - beta2^step
__global__ void adam_kernel(float *__restrict__ theta, const float *__restrict__ grad, float *__restrict__ m,
                            float *__restrict__ v, int P, double lr, double beta1, double beta2, double eps,
                            double corr1, double corr2)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    const double g = (double)grad[p];
    const double mn = beta1 * (double)m[p] + (1.0 - beta1) * g;
    const double vn = beta2 * (double)v[p] + (1.0 - beta2) * g * g;
    m[p] = (float)mn;
    v[p] = (float)vn;
    theta[p] = (float)((double)theta[p] - lr * (mn / corr1) / (sqrt(vn / corr2) + eps));
}

policy_args make_pargs(const bagel_ctx *c, int slot)
{
    policy_args a;
    a.B = c->dm.B; a.nl = c->n_layers; a.ds = c->dm.d_s;
    for (int i = 0; i < 4; ++i) a.width[i] = c->width[i];
    for (int i = 0; i < 3; ++i) {
        a.b_off[i] = c->b_off[i];
        a.wp_off[i] = c->wpf_off[i];
        a.kp[i] = c->wpf_kp[i];
        a.rp[i] = c->wpf_rp[i];
    }
    a.act_bound = c->dm.act_bound;
    const size_t B = c->dm.B;
    for (int l = 0; l < 3; ++l) a.h[l] = (l < c->n_layers) ? c->tape_h[l] + (size_t)slot * c->width[l] * B : nullptr;
    a.a_slot = c->tape_a + (size_t)slot * c->dm.d_a * B;
    a.xbuf = c->xbuf;
    a.theta = nullptr;
    a.Wp = c->wpad_f;
    return a;
}

}  // namespace

hipError_t bagel_launch_pack_theta(bagel_ctx *c, const float *theta)
{
    for (int l = 0; l < c->n_layers; ++l) {
        const int no = c->width[l + 1], ni = c->width[l];
        const int nf = c->wpf_rp[l] * c->wpf_kp[l], nb = c->wpb_rp[l] * c->wpb_kp[l];
        const int n = nf > nb ? nf : nb;
        hipLaunchKernelGGL(pack_theta_kernel, dim3((n + 255) / 256), dim3(256), 0, c->stream, theta, c->wpad_f,
                           c->wpad_b, no, ni, c->w_off[l], c->wpf_off[l], c->wpf_rp[l], c->wpf_kp[l], c->wpb_off[l],
                           c->wpb_rp[l], c->wpb_kp[l]);
    }
    return hipGetLastError();
}

hipError_t bagel_launch_policy_forward(bagel_ctx *c, int slot, const float *theta)
{
    policy_args a = make_pargs(c, slot);
    a.theta = theta;
    hipLaunchKernelGGL(policy_forward_kernel, dim3((c->dm.B + PL - 1) / PL), dim3(PW * 64), 0, c->stream, a);
    return hipGetLastError();
}

hipError_t bagel_launch_step_tail(bagel_ctx *c, int t, int slot, int next_slot, bool jac, bool add_cost,
                                  bool write_tape_s, const float *theta, const float *goals, float *states_out,
                                  bool direct)
{
    const size_t B = c->dm.B;
    const bool has_next = t + 1 < c->dm.H && next_slot >= 0;
    tail_args r;
    r.D = c->D; r.M = c->M; r.dg = c->dm.d_g;
    r.ngk = (c->nck + 3) / 4; r.ngl = (c->ncl + 3) / 4;
    r.ncomp = jac ? 1 + c->D : 1;
    r.cost_kind = c->dm.cost_kind; r.add_cost = add_cost ? 1 : 0; r.do_policy = has_next ? 1 : 0;
    r.direct = direct ? 1 : 0;
    r.sigma_r = c->dm.sigma_r;
    for (int j = 0; j < 8; ++j) { r.tracked[j] = c->dm.tracked[j]; r.q[j] = c->dm.q[j]; }
    r.A = c->A; r.amp = c->amp; r.part = c->part; r.lpt = c->lpt;
    r.x_cur = c->xbuf; r.x_next = c->xbuf_alt;
    r.tape_s_next = write_tape_s ? c->tape_s + (size_t)(t + 1) * c->dm.d_s * B : nullptr;
    r.states_out_next = states_out ? states_out + (size_t)(t + 1) * B * c->dm.d_s : nullptr;
    r.goals_t = goals + (size_t)t * B * c->dm.d_g;
    r.goals_next = has_next ? goals + (size_t)(t + 1) * B * c->dm.d_g : nullptr;
    r.jdst = (jac && direct) ? c->tape_J + (size_t)slot * c->M * c->D * B : nullptr;
    policy_args a = make_pargs(c, has_next ? next_slot : 0);
    a.theta = theta;
    a.xbuf = c->xbuf_alt;              // the action of step t+1 joins s_{t+1}
    hipLaunchKernelGGL(step_tail_kernel, dim3((c->dm.B + PL - 1) / PL), dim3(PW * 64), 0, c->stream, r, a);
    return hipGetLastError();
}

hipError_t bagel_launch_policy_replay(bagel_ctx *c, int t0, int t1, const float *theta, const float *goals)
{
    policy_args a = make_pargs(c, 0);
    a.theta = theta;
    replay_args r;
    r.tape_s = c->tape_s; r.goals = goals; r.t0 = t0; r.dg = c->dm.d_g; r.n_slots = t1 - t0;
    hipLaunchKernelGGL(policy_replay_kernel, dim3((c->dm.B + PL - 1) / PL, (t1 - t0 + REPLAY_SLOTS - 1) / REPLAY_SLOTS),
                       dim3(PW * 64), 0, c->stream, a, r);
    return hipGetLastError();
}

hipError_t bagel_launch_backward_sweep(bagel_ctx *c, int t_lo, int t_hi, const float *goals, float *grad_s0)
{
    sweep_args a;
    a.B = c->dm.B; a.nl = c->n_layers; a.ds = c->dm.d_s; a.da = c->dm.d_a; a.dg = c->dm.d_g; a.D = c->D; a.M = c->M;
    a.H = c->dm.H; a.t_hi = t_hi; a.t_lo = t_lo;
    for (int i = 0; i < 4; ++i) a.width[i] = c->width[i];
    for (int l = 0; l < 3; ++l) {
        a.wp_off[l] = c->wpb_off[l];
        a.kp[l] = c->wpb_kp[l];
        a.tape_h[l] = l < c->n_layers ? c->tape_h[l] : nullptr;
        a.tape_d[l] = l < c->n_layers ? c->tape_d[l] : nullptr;
    }
    a.act_bound = c->dm.act_bound; a.cost_kind = c->dm.cost_kind; a.sigma_r = c->dm.sigma_r;
    for (int j = 0; j < 8; ++j) { a.tracked[j] = c->dm.tracked[j]; a.q[j] = c->dm.q[j]; }
    a.Wp = c->wpad_b;
    // the Jacobian tape spans the whole horizon when the activation tape is kept per segment
    const bool per_segment = c->T_tape < c->dm.H;
    a.tape_a = c->tape_a; a.tape_s = c->tape_s;
    a.tape_J = c->tape_J + (per_segment ? (size_t)t_lo * c->M * c->D * c->dm.B : 0);
    a.goals = goals; a.lam = c->lam; a.grad_s0 = grad_s0;
    hipLaunchKernelGGL(backward_sweep_kernel, dim3((c->dm.B + PL - 1) / PL), dim3(PW * 64), 0, c->stream, a);
    return hipGetLastError();
}

hipError_t bagel_launch_adam(bagel_ctx *c, float *theta, const float *grad, float *m, float *v, int count, double lr,
                             double beta1, double beta2, double eps, double corr1, double corr2)
{
    hipLaunchKernelGGL(adam_kernel, dim3((count + 255) / 256), dim3(256), 0, c->stream, theta, grad, m, v, count, lr,
                       beta1, beta2, eps, corr1, corr2);
    return hipGetLastError();
}

namespace {
template <int WA, int WB, int TA, int TB, int NST>
hipError_t launch_wg_tiled(bagel_ctx *c, int which, int nz, int l, int no, int ni, int B, int n_slots, int per_t)
{
    using T = wg_tiling<WA, WB, TA, TB, NST>;
    auto kernel = weight_grad_tiled_kernel<WA, WB, TA, TB, NST>;
    if (!(c->wg_lds_raised & (1 << which))) {       // a per-device function attribute: set once per context
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)T::LDS_BYTES);
        if (e != hipSuccess) return e;
        c->wg_lds_raised |= 1 << which;
    }
    hipLaunchKernelGGL(kernel, dim3(nz), dim3(64 * T::NW), T::LDS_BYTES, c->stream, c->tape_d[l], c->tape_h[l], c->gsplit,
                       no, ni, B, n_slots, per_t, c->w_off[l], c->b_off[l], c->P);
    return hipGetLastError();
}
}  // namespace

hipError_t bagel_launch_weight_grad(bagel_ctx *c, int n_slots, bool accumulate, float *grad_theta)
{
    const int B = c->dm.B;
    const int chunks_per_slot = (B + 7) / 8;
    const int total = n_slots * chunks_per_slot;
    const int ksplit = total < c->ksplit ? total : c->ksplit;
    const int per = (total + ksplit - 1) / ksplit;
    const int nz = (total + per - 1) / per;
    for (int l = 0; l < c->n_layers; ++l) {
        const int no = c->width[l + 1], ni = c->width[l];
        if (B % WG_KC == 0 && no <= 256 && ni <= 256) {
            // operands staged through LDS: the wide layer (both sides above 128) and the skinny ones
            // (one side of at most 32, the other above 128)
            const int tiles = n_slots * (B / WG_KC);
            const int per_t = (tiles + nz - 1) / nz;
            hipError_t e = hipSuccess;
            bool done = true;
            if (no > 128 && ni > 128)
                e = launch_wg_tiled<4, 4, 2, 2, 2>(c, 0, nz, l, no, ni, B, n_slots, per_t);
            else if (no > 128 && ni <= 32)
                e = launch_wg_tiled<8, 1, 1, 1, 3>(c, 1, nz, l, no, ni, B, n_slots, per_t);
            else if (no <= 32 && ni > 128)
                e = launch_wg_tiled<1, 8, 1, 1, 3>(c, 2, nz, l, no, ni, B, n_slots, per_t);
            else
                done = false;
            if (e != hipSuccess) return e;
            if (done) continue;
        }
        dim3 grid(nz, (no + 255) / 256, (ni + 255) / 256);
        const int wrows = no >= 256 ? 4 : (no + 63) / 64, wcols = ni >= 256 ? 4 : (ni + 63) / 64;
        if (B % 8 == 0)
            hipLaunchKernelGGL(weight_grad_kernel<true>, grid, dim3(64 * wrows * wcols), 0, c->stream, c->tape_d[l],
                               c->tape_h[l], c->gsplit, no, ni, B, n_slots, chunks_per_slot, per, c->w_off[l],
                               c->b_off[l], c->P, wcols);
        else
            hipLaunchKernelGGL(weight_grad_kernel<false>, grid, dim3(64 * wrows * wcols), 0, c->stream, c->tape_d[l],
                               c->tape_h[l], c->gsplit, no, ni, B, n_slots, chunks_per_slot, per, c->w_off[l],
                               c->b_off[l], c->P, wcols);
    }
    hipLaunchKernelGGL(grad_reduce_kernel, dim3((c->P + 63) / 64), dim3(256), 0, c->stream, c->gsplit, c->gacc, c->P,
                       nz, accumulate, grad_theta);
    return hipGetLastError();
}
