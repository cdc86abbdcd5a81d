// fp32-activation path: plain LDS-tiled FMA kernels.  It exists for the small all-fp32 configuration
// (parity to 1e-5); throughput is not its purpose.  Every quantisation decision here uses the exact
// binary32 quotient.
#include "common.h"
#include "kernels.h"

namespace eqat {

// ---- element accessors (return 0 outside the matrix) ----------------------------------------------
struct PlainF32 {          // M[r][c], row-major, ld = columns
    const float *p; int rows, cols;
    __device__ __forceinline__ float at(int r, int c) const { return (r < rows && c < cols) ? p[(size_t)r * cols + c] : 0.0f; }
};

template <typename WT> struct FakeQuantW {   // What[o][i] from W, s, z  (Eqs.(1),(2))
    const WT *W; const float *s, *z; int O, I, g, G; float qmax;
    __device__ __forceinline__ float at(int o, int i) const
    {
        if (o >= O || i >= I) return 0.0f;
        const int j = i / g;
        const float sv = s[(size_t)o * G + j], zb = zbar_of(z[(size_t)o * G + j], qmax);
        const float r = __builtin_rintf(to_float(W[(size_t)o * I + i]) / sv);
        const float q = __builtin_fminf(__builtin_fmaxf(r + zb, 0.0f), qmax);
        return (q - zb) * sv;
    }
};

template <int BITS> struct PackedW {         // What[o][i] from packed codes and (s, z) pairs  (Eq.(2))
    const uint32_t *codes; const floatx2 *sz; int O, I, g, G;
    __device__ __forceinline__ float at(int o, int i) const
    {
        if (o >= O || i >= I) return 0.0f;
        const floatx2 p = sz[(size_t)o * G + i / g];
        const uint32_t *seg = codes + ((size_t)o * I + (i & ~31)) / 32 * BITS;
        return ((float)code_at_rt<BITS>(seg, i & 31) - p[1]) * p[0];
    }
};

// C[m][n] = sum_k A(m,k) * B(k,n);  A is read through (TRANS_A ? a.at(k,m) : a.at(m,k)),
// B through (TRANS_B ? b.at(n,k) : b.at(k,n)).  64x64 tile, 16x16 threads, 4x4 outputs per thread.
template <typename AccA, typename AccB, bool TRANS_A, bool TRANS_B>
__global__ __launch_bounds__(256) void k_f32_gemm(AccA a, AccB b, float *__restrict__ C, int M, int N, int K)
{
    __shared__ float As[16][64 + 1];
    __shared__ float Bs[16][64 + 1];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int e = threadIdx.x; e < 16 * 64; e += 256) {
            // consecutive threads walk the contiguous axis of each operand
            int kk, mm;
            if (TRANS_A) { mm = e & 63; kk = e >> 6; } else { kk = e & 15; mm = e >> 4; }
            As[kk][mm] = (k0 + kk < K) ? (TRANS_A ? a.at(k0 + kk, m0 + mm) : a.at(m0 + mm, k0 + kk)) : 0.0f;
            int kb, nn;
            if (TRANS_B) { kb = e & 15; nn = e >> 4; } else { nn = e & 63; kb = e >> 6; }
            Bs[kb][nn] = (k0 + kb < K) ? (TRANS_B ? b.at(n0 + nn, k0 + kb) : b.at(k0 + kb, n0 + nn)) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { av[i] = As[kk][ty * 4 + i]; bv[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) C[(size_t)m * N + n] = acc[i][j];
        }
}

// Per-group epilogue of the Block-AP backward (Eqs.(3)-(5)): one thread per (o, j).
template <typename WT>
__global__ __launch_bounds__(256) void k_f32_epilogue_block_ap(const float *__restrict__ dwhat, const WT *__restrict__ W,
                                                               const float *__restrict__ s, const float *__restrict__ z,
                                                               WT *__restrict__ dW, float *__restrict__ ds, float *__restrict__ dz,
                                                               int O, int I, int g, int G, float qmax)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= O * G) return;
    const int o = t / G, j = t - o * G;
    const float sv = s[t], zb = zbar_of(z[t], qmax);
    float gs = 0.0f, gz = 0.0f;
    for (int i = j * g; i < (j + 1) * g; ++i) {
        const size_t e = (size_t)o * I + i;
        const float d = dwhat[e];
        const float tq = to_float(W[e]) / sv;
        const float r = __builtin_rintf(tq);
        const float qpre = r + zb;
        float cs, cw;
        if (qpre < 0.0f)       { cs = -zb;        gz += d; cw = 0.0f; }
        else if (qpre > qmax)  { cs = qmax - zb;  gz += d; cw = 0.0f; }
        else                   { cs = r - tq;              cw = 1.0f; }
        gs = __builtin_fmaf(d, cs, gs);
        if (dW != nullptr) dW[e] = (WT)(d * cw);
    }
    if (ds != nullptr) ds[t] = gs;
    if (dz != nullptr) dz[t] = -sv * gz;
}

template <int BITS>
__global__ __launch_bounds__(256) void k_f32_epilogue_e2e(const float *__restrict__ dwhat, const uint32_t *__restrict__ codes,
                                                          const floatx2 *__restrict__ sz, float *__restrict__ ds,
                                                          float *__restrict__ dz, int O, int I, int g, int G)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= O * G) return;
    const int o = t / G, j = t - o * G;
    const float zq = sz[t][1];
    float gs = 0.0f, gz = 0.0f;
    for (int i = j * g; i < (j + 1) * g; ++i) {
        const size_t e = (size_t)o * I + i;
        const uint32_t *seg = codes + (e & ~(size_t)31) / 32 * BITS;
        gs = __builtin_fmaf(dwhat[e], (float)code_at_rt<BITS>(seg, i & 31) - zq, gs);
        gz += dwhat[e];
    }
    if (ds != nullptr) ds[t] = gs;
    if (dz != nullptr) dz[t] = -sz[t][0] * gz;
}

// ---- host ------------------------------------------------------------------------------------------
template <typename AccA, typename AccB, bool TA, bool TB>
static void gemm(AccA a, AccB b, float *C, int M, int N, int K, hipStream_t st)
{
    if (M <= 0 || N <= 0) return;
    const dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
    k_f32_gemm<AccA, AccB, TA, TB><<<grid, block, 0, st>>>(a, b, C, M, N, K);
}

template <bool DX, typename AccW>
static void fwd_or_dx(const Problem &p, const void *A, AccW w, void *out, hipStream_t st)
{
    if (!DX) gemm<PlainF32, AccW, false, true>(PlainF32{(const float *)A, (int)p.T, (int)p.I}, w, (float *)out, (int)p.T, (int)p.O, (int)p.I, st);
    else     gemm<PlainF32, AccW, false, false>(PlainF32{(const float *)A, (int)p.T, (int)p.O}, w, (float *)out, (int)p.T, (int)p.I, (int)p.O, st);
}

template <bool DX>
static void dispatch_w(const Problem &p, bool packed, const void *A, const void *Wc, const float *s, const void *zsz, void *out, hipStream_t st)
{
    const int O = (int)p.O, I = (int)p.I, g = (int)p.g, G = (int)p.G;
    if (packed) {
        const uint32_t *c = (const uint32_t *)Wc; const floatx2 *sz = (const floatx2 *)zsz;
        if (p.bits == 2) fwd_or_dx<DX>(p, A, PackedW<2>{c, sz, O, I, g, G}, out, st);
        else if (p.bits == 3) fwd_or_dx<DX>(p, A, PackedW<3>{c, sz, O, I, g, G}, out, st);
        else fwd_or_dx<DX>(p, A, PackedW<4>{c, sz, O, I, g, G}, out, st);
    } else {
        const float qmax = (float)((1 << p.bits) - 1);
        if (p.w_bf16) fwd_or_dx<DX>(p, A, FakeQuantW<bf16_t>{(const bf16_t *)Wc, s, (const float *)zsz, O, I, g, G, qmax}, out, st);
        else fwd_or_dx<DX>(p, A, FakeQuantW<float>{(const float *)Wc, s, (const float *)zsz, O, I, g, G, qmax}, out, st);
    }
}

void launch_f32_fwd(const Problem &p, bool packed, const void *X, const void *Wc, const float *s, const void *zsz, void *Y, hipStream_t st)
{
    dispatch_w<false>(p, packed, X, Wc, s, zsz, Y, st);
}
void launch_f32_dx(const Problem &p, bool packed, const void *dY, const void *Wc, const float *s, const void *zsz, void *dX, hipStream_t st)
{
    dispatch_w<true>(p, packed, dY, Wc, s, zsz, dX, st);
}

void launch_f32_dw(const Problem &p, bool block_ap, const void *X, const void *dY, const void *Wc, const float *s,
                   const void *zsz, float *dwhat, void *dW, float *ds, float *dz, hipStream_t st)
{
    const int O = (int)p.O, I = (int)p.I, g = (int)p.g, G = (int)p.G, T = (int)p.T;
    // dWhat[o][i] = sum_t dY[t][o] * X[t][i]
    gemm<PlainF32, PlainF32, true, false>(PlainF32{(const float *)dY, T, O}, PlainF32{(const float *)X, T, I}, dwhat, O, I, T, st);
    const dim3 grid((unsigned)(((size_t)O * G + 255) / 256)), block(256);
    if (block_ap) {
        const float qmax = (float)((1 << p.bits) - 1);
        if (p.w_bf16) k_f32_epilogue_block_ap<bf16_t><<<grid, block, 0, st>>>(dwhat, (const bf16_t *)Wc, s, (const float *)zsz, (bf16_t *)dW, ds, dz, O, I, g, G, qmax);
        else k_f32_epilogue_block_ap<float><<<grid, block, 0, st>>>(dwhat, (const float *)Wc, s, (const float *)zsz, (float *)dW, ds, dz, O, I, g, G, qmax);
    } else {
        const uint32_t *c = (const uint32_t *)Wc; const floatx2 *sz = (const floatx2 *)zsz;
        if (p.bits == 2) k_f32_epilogue_e2e<2><<<grid, block, 0, st>>>(dwhat, c, sz, ds, dz, O, I, g, G);
        else if (p.bits == 3) k_f32_epilogue_e2e<3><<<grid, block, 0, st>>>(dwhat, c, sz, ds, dz, O, I, g, G);
        else k_f32_epilogue_e2e<4><<<grid, block, 0, st>>>(dwhat, c, sz, ds, dz, O, I, g, G);
    }
}

}  // namespace eqat
