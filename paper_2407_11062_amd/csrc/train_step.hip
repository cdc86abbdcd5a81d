// Block-AP step glue (Sec. 3.2: a block is trained against its full-precision counterpart with a reconstruction loss;
// Sec. 4.1 "Training": one learning rate for the quantization parameters, another for the weights).  The paper names
// neither the loss form nor the optimizer; mean squared error and AdamW are taken.  Both kernels are streaming passes
// bound by HBM: 8 elements per lane and access, 16-byte loads and stores, all arithmetic in binary32.
#include "common.h"
#include "kernels.h"

namespace eqat {
namespace {

constexpr int kThreads = 256;
constexpr int kLossBlocksMax = 2048;    // partial sums of the loss; also the length of the workspace in floats

__device__ __forceinline__ void load8(const float *p, float (&v)[8])
{
    const floatx4 a = reinterpret_cast<const floatx4 *>(p)[0], b = reinterpret_cast<const floatx4 *>(p)[1];
#pragma unroll
    for (int k = 0; k < 4; ++k) { v[k] = a[k]; v[4 + k] = b[k]; }
}
__device__ __forceinline__ void load8(const bf16_t *p, float (&v)[8])
{
    const uintx4 u = *reinterpret_cast<const uintx4 *>(p);
#pragma unroll
    for (int k = 0; k < 4; ++k) { v[2 * k] = __uint_as_float(u[k] << 16); v[2 * k + 1] = __uint_as_float(u[k] & 0xFFFF0000u); }
}
__device__ __forceinline__ void store8(float *p, const float (&v)[8])
{
    floatx4 a, b;
#pragma unroll
    for (int k = 0; k < 4; ++k) { a[k] = v[k]; b[k] = v[4 + k]; }
    reinterpret_cast<floatx4 *>(p)[0] = a;
    reinterpret_cast<floatx4 *>(p)[1] = b;
}
__device__ __forceinline__ void store8(bf16_t *p, const float (&v)[8])
{
    bf16x8 o;
#pragma unroll
    for (int k = 0; k < 8; ++k) o[k] = (bf16_t)v[k];          // round to nearest even
    *reinterpret_cast<bf16x8 *>(p) = o;
}
__device__ __forceinline__ void store1(float *p, float v) { *p = v; }
__device__ __forceinline__ void store1(bf16_t *p, float v) { *p = (bf16_t)v; }

// Sum over the workgroup in a fixed order (lanes by xor butterfly, then the waves in order); valid in thread 0.
__device__ __forceinline__ float block_sum(float v)
{
    __shared__ float wave_sum[kThreads / 64];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) t += wave_sum[w];
    }
    return t;
}

// partial[b] = sum over the elements of workgroup b of (Y - Yref)^2;  dY = (Y - Yref) * two_over_n  (dY may be NULL)
template <typename T>
__global__ __launch_bounds__(kThreads) void k_recon_loss(const T *__restrict__ Y, const T *__restrict__ R, T *__restrict__ dY,
                                                         float *__restrict__ partial, int64_t n, float two_over_n)
{
    const int64_t n8 = n >> 3;
    float acc = 0.f;
    for (int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x; c < n8; c += (int64_t)gridDim.x * kThreads) {
        float y[8], r[8];
        load8(Y + 8 * c, y);
        load8(R + 8 * c, r);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            y[k] -= r[k];
            acc = fmaf(y[k], y[k], acc);
            y[k] *= two_over_n;
        }
        if (dY != nullptr) store8(dY + 8 * c, y);
    }
    // the last n % 8 elements: one each for the first lanes of workgroup 0
    if (blockIdx.x == 0 && (int64_t)threadIdx.x < (n & 7)) {
        const int64_t e = 8 * n8 + threadIdx.x;
        const float d = to_float(Y[e]) - to_float(R[e]);
        acc = fmaf(d, d, acc);
        if (dY != nullptr) store1(dY + e, d * two_over_n);
    }
    const float t = block_sum(acc);
    if (threadIdx.x == 0) partial[blockIdx.x] = t;
}

// loss = (sum of the partials, in a fixed order) / n
__global__ __launch_bounds__(kThreads) void k_recon_finish(const float *__restrict__ partial, int n_partial, float *__restrict__ loss,
                                                           float inv_n)
{
    float acc = 0.f;
    for (int k = threadIdx.x; k < n_partial; k += kThreads) acc += partial[k];
    const float t = block_sum(acc);
    if (threadIdx.x == 0) loss[0] = t * inv_n;
}

// ---- AdamW ---------------------------------------------------------------------------------------------------------
struct AdamSeg {
    void *p; const void *g; float *m; float *v;
    int64_t n;
    float lr, decay;                    // decay = lr * weight_decay
    float p_min;                        // the updated parameter is held at or above this (-inf: no bound)
    uint32_t first_block;
    int32_t bf16;                       // dtype of p and g
};
struct AdamArgs {
    AdamSeg seg[3];                     // W, s, z (n = 0: absent)
    float b1, b2, omb1, omb2, eps, c1, c2;   // omb = 1 - b;  c1 = 1 / (1 - b1^step), c2 = 1 / (1 - b2^step)
};

__device__ __forceinline__ void adam_one(float &p, float g, float &m, float &v, const AdamSeg &sg, const AdamArgs &a)
{
    p -= sg.decay * p;
    m = a.b1 * m + a.omb1 * g;
    v = a.b2 * v + a.omb2 * g * g;
    p -= sg.lr * (m * a.c1) / (sqrtf(v * a.c2) + a.eps);
    p = fmaxf(p, sg.p_min);
}

template <typename T>
__device__ __forceinline__ void adam_chunk(const AdamSeg &sg, const AdamArgs &a, int64_t c)
{
    T *P = static_cast<T *>(sg.p);
    const T *G = static_cast<const T *>(sg.g);
    const int64_t e0 = 8 * c;
    if (e0 + 8 <= sg.n) {
        float p[8], g[8], m[8], v[8];
        load8(P + e0, p); load8(G + e0, g); load8(sg.m + e0, m); load8(sg.v + e0, v);
#pragma unroll
        for (int k = 0; k < 8; ++k) adam_one(p[k], g[k], m[k], v[k], sg, a);
        store8(P + e0, p); store8(sg.m + e0, m); store8(sg.v + e0, v);
    } else {
        for (int64_t e = e0; e < sg.n; ++e) {
            float p = to_float(P[e]), m = sg.m[e], v = sg.v[e];
            adam_one(p, to_float(G[e]), m, v, sg, a);
            store1(P + e, p); sg.m[e] = m; sg.v[e] = v;
        }
    }
}

// One launch updates the weights, the step sizes and the zero points of a linear: workgroups
// [seg[i].first_block, seg[i+1].first_block) own parameter group i, 8 elements per lane.
__global__ __launch_bounds__(kThreads) void k_adamw(AdamArgs a)
{
    const int si = blockIdx.x >= a.seg[2].first_block ? 2 : blockIdx.x >= a.seg[1].first_block ? 1 : 0;
    const AdamSeg sg = si == 2 ? a.seg[2] : si == 1 ? a.seg[1] : a.seg[0];     // selects, not a dynamic index
    const int64_t c = (int64_t)(blockIdx.x - sg.first_block) * kThreads + threadIdx.x;
    if (8 * c >= sg.n) return;
    if (sg.bf16) adam_chunk<bf16_t>(sg, a, c);
    else adam_chunk<float>(sg, a, c);
}

inline uint32_t blocks_for(int64_t n) { return (uint32_t)((n + 8 * kThreads - 1) / (8 * kThreads)); }

}  // namespace

size_t recon_loss_ws_bytes() { return (size_t)kLossBlocksMax * sizeof(float); }

void launch_recon_loss(int64_t n, bool bf16, const void *Y, const void *Yref, float *loss, void *dY, float *partial,
                       hipStream_t st)
{
    const int64_t want = (n / 8 + kThreads - 1) / kThreads;
    const int nb = (int)(want < 1 ? 1 : want > kLossBlocksMax ? kLossBlocksMax : want);
    const float two_over_n = (float)(2.0 / (double)n), inv_n = (float)(1.0 / (double)n);
    if (bf16)
        hipLaunchKernelGGL(k_recon_loss<bf16_t>, dim3(nb), dim3(kThreads), 0, st, static_cast<const bf16_t *>(Y),
                           static_cast<const bf16_t *>(Yref), static_cast<bf16_t *>(dY), partial, n, two_over_n);
    else
        hipLaunchKernelGGL(k_recon_loss<float>, dim3(nb), dim3(kThreads), 0, st, static_cast<const float *>(Y),
                           static_cast<const float *>(Yref), static_cast<float *>(dY), partial, n, two_over_n);
    hipLaunchKernelGGL(k_recon_finish, dim3(1), dim3(kThreads), 0, st, partial, nb, loss, inv_n);
}

void launch_adamw(const AdamGroup *groups, float beta1, float beta2, float eps, int step, hipStream_t st)
{
    AdamArgs a{};
    uint32_t first = 0;
    for (int i = 0; i < 3; ++i) {
        const AdamGroup &gr = groups[i];
        AdamSeg &sg = a.seg[i];
        sg.p = gr.p; sg.g = gr.g; sg.m = gr.m; sg.v = gr.v;
        sg.n = gr.p != nullptr ? gr.n : 0;
        sg.lr = gr.lr; sg.decay = (float)((double)gr.lr * (double)gr.weight_decay);
        sg.first_block = first; sg.bf16 = gr.bf16 ? 1 : 0; sg.p_min = gr.p_min;
        first += blocks_for(sg.n);
    }
    if (first == 0) return;
    a.b1 = beta1; a.b2 = beta2; a.omb1 = (float)(1.0 - (double)beta1); a.omb2 = (float)(1.0 - (double)beta2); a.eps = eps;
    a.c1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
    a.c2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
    hipLaunchKernelGGL(k_adamw, dim3(first), dim3(kThreads), 0, st, a);
}

}  // namespace eqat
