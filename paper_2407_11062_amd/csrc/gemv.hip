// E2E-QP forward for a handful of tokens (decode-time matrix-vector product, App. "Speedup with BitBLAS" of the paper
// measures this shape of work):  Y[t,o] = sum_i X[t,i] * (w_q[o,i] - z[o,j]) * s[o,j],  T <= 16.
//
// HBM-bound: every weight is read once, N/8 bytes, straight from the dense packed stream of the C ABI (no re-layout
// pass, which would triple the traffic).  One workgroup owns 16 output rows; its 4 waves split the input dimension
// and meet in LDS at the end (fixed order: deterministic).  The contraction runs on v_mfma_f32_16x16x32_bf16 with
// the WEIGHTS as the A operand (16 rows x 32 k) and the tokens as the 16 columns of B, so that one byte-permute table
// per 32-code segment (WhatTable, shared with the GEMM producer) turns codes into bf16 at about one VALU
// instruction per weight and the multiply-adds cost nothing.
//
// Order of the contraction index.  A lane holds one 32-code segment of one row and feeds 8 of its codes to each of 4
// MFMAs.  In the dense 2- and 4-bit streams, (word >> shift) & 0x03030303 / 0x0F0F0F0F leaves four codes that are 4
// (resp. 2) apart, not consecutive, in the four bytes of a register.  MFMA does not care in which order k runs as long
// as both operands agree, so the token rows are staged in LDS once per workgroup in exactly that order (slot_code()).
// The dense 3-bit stream has no byte alignment at all; its codes are extracted one by one (slower, still correct).
#include "common.h"
#include "kernels.h"

#include <algorithm>

namespace eqat {

namespace {

// code index (0..31, within a segment) that sits in contraction slot m (0..7) of MFMA t (0..3) of the lane owning the segment
template <int BITS> __host__ __device__ constexpr int slot_code(int t, int m)
{
    if (BITS == 2) return 16 * (t / 2) + 4 * (m % 4) + (2 * (t % 2) + m / 4);
    if (BITS == 4) return 8 * t + 2 * (m % 4) + m / 4;
    return 8 * t + m;
}

// inverse of slot_code: position (8 t + m) of code c in the slot order of its segment
template <int BITS> __host__ __device__ constexpr int code_slot(int c)
{
    if (BITS == 2) { const int wd = c / 16, k = c % 16, p = k % 4, q = k / 4; return 8 * (2 * wd + p / 2) + 4 * (p % 2) + q; }
    if (BITS == 4) { const int t = c / 8, k = c % 8, p = k % 2, q = k / 2; return 8 * t + 4 * p + q; }
    return c;
}

template <int BITS> constexpr bool slot_maps_are_inverse()
{
    for (int c = 0; c < 32; ++c) {
        const int sl = code_slot<BITS>(c);
        if (sl < 0 || sl >= 32 || slot_code<BITS>(sl / 8, sl % 8) != c) return false;
    }
    return true;
}
static_assert(slot_maps_are_inverse<2>() && slot_maps_are_inverse<3>() && slot_maps_are_inverse<4>(), "slot order");

// the 8 weights of MFMA t of a segment, in slot order
template <int BITS, int T4>
__device__ __forceinline__ bf16x8 eight_of(const WhatTable<BITS> &tab, const CodeWords<BITS> &c)
{
    uint32_t t0, t1;
    if constexpr (BITS == 2) {
        const uint32_t w = c.w[T4 / 2];
        t0 = (w >> (2 * (2 * (T4 % 2) + 0))) & 0x03030303u;
        t1 = (w >> (2 * (2 * (T4 % 2) + 1))) & 0x03030303u;
    } else if constexpr (BITS == 4) {
        const uint32_t w = c.w[T4];
        t0 = w & 0x0F0F0F0Fu;
        t1 = (w >> 4) & 0x0F0F0F0Fu;
    } else {
        t0 = code_at<3, 8 * T4 + 0>(c) | (code_at<3, 8 * T4 + 1>(c) << 8) | (code_at<3, 8 * T4 + 2>(c) << 16) | (code_at<3, 8 * T4 + 3>(c) << 24);
        t1 = code_at<3, 8 * T4 + 4>(c) | (code_at<3, 8 * T4 + 5>(c) << 8) | (code_at<3, 8 * T4 + 6>(c) << 16) | (code_at<3, 8 * T4 + 7>(c) << 24);
    }
    uintx4 u;
    uint32_t d0, d1;
    tab.four(t0, d0, d1); u[0] = d0; u[1] = d1;
    tab.four(t1, d0, d1); u[2] = d0; u[3] = d1;
    return __builtin_bit_cast(bf16x8, u);
}

struct GemvArgs {
    const bf16_t *X; const uint32_t *Wp; const float *s; const uint32_t *zp; const float *zf; bf16_t *Y;
    int T, I, O, G, g;
    uint32_t spg_magic;            // ceil(2^32 / (g/32)): group of segment sg = mulhi(sg, spg_magic), exact for sg * (g/32) < 2^32
    uint32_t w_row_bytes, z_row_words;
    uint32_t w_bytes, s_bytes, z_bytes;
};

constexpr int kGemvRows = 16;      // output rows per workgroup (the M of the MFMA)
constexpr int kGemvWaves = 4;      // waves per workgroup, splitting the input dimension
constexpr int kGemvMaxWaves = 8;   // ... of the run kernel when it is launched with one wave per run
constexpr int kGemvUnroll = 4;     // chunks (4 segments = 128 inputs each) in flight per wave

// General group sizes: step size and zero point fetched per 32-code segment (many small scattered loads: slow, kept for
// group sizes the run kernel below does not take).  RB = 16-row blocks per workgroup.
template <int BITS, bool FLOATZ, int RB>
__global__ __launch_bounds__(64 * kGemvWaves) void k_gemv_any(const GemvArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t *xs = reinterpret_cast<bf16_t *>(smem_raw);                       // [T][I], contraction-slot order
    float *red = reinterpret_cast<float *>(smem_raw);                        // reused after the loop: [waves][RB][16][16]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, kq = lane >> 4;
    const int n_segs = a.I >> 5;

    // ---- stage the token rows in slot order: one 32-input segment per thread and trip, 2-byte LDS scatter with
    //      compile-time offsets
    for (int e = tid; e < a.T * n_segs; e += 64 * kGemvWaves) {
        const int n = e / n_segs, seg = e - n * n_segs;
        const bf16_t *src = a.X + (size_t)n * a.I + seg * 32;
        bf16_t *dst = xs + (size_t)n * a.I + seg * 32;
        bf16x8 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const bf16x8 *>(src + 8 * q);
#pragma unroll
        for (int c = 0; c < 32; ++c) dst[code_slot<BITS>(c)] = v[c / 8][c % 8];
    }
    __syncthreads();

    const __amdgpu_buffer_rsrc_t rW = make_rsrc(a.Wp, a.w_bytes);
    const __amdgpu_buffer_rsrc_t rS = make_rsrc(a.s, a.s_bytes);
    const __amdgpu_buffer_rsrc_t rZ = make_rsrc(FLOATZ ? (const void *)a.zf : (const void *)a.zp, a.z_bytes);
    int o[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) o[rb] = (blockIdx.x * RB + rb) * kGemvRows + r;
    // The waves interleave: in trip `it` wave w takes chunks [(it * waves + w) * unroll, +unroll), so that one trip of the
    // workgroup reads waves * unroll * 128 codes = one contiguous run of every row (DRAM page locality).
    const int n_chunks = (a.I + 127) / 128;
    const int c_begin = wave * kGemvUnroll, c_end = n_chunks;
    // lanes whose column is not a token multiply token 0 again; their columns of the result are never stored
    const bf16_t *xlane = xs + (size_t)((lane & 15) < a.T ? (lane & 15) : 0) * a.I;

    floatx4 acc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

    for (int c0 = c_begin; c0 < c_end; c0 += kGemvUnroll * kGemvWaves) {
        CodeWords<BITS> cw[kGemvUnroll][RB];
        float sv[kGemvUnroll][RB], zv[kGemvUnroll][RB];
        uint32_t zw0[kGemvUnroll][RB], zw1[kGemvUnroll][RB];
        // all loads of the unrolled chunks first
#pragma unroll
        for (int u = 0; u < kGemvUnroll; ++u) {
            const int seg = (c0 + u) * 4 + kq;
            const uint32_t j = a.spg_magic ? __umulhi((uint32_t)seg, a.spg_magic) : (uint32_t)seg;      // 0: one segment per group
            const bool seg_ok = (c0 + u) < c_end && seg < n_segs;
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const bool ok = seg_ok && o[rb] < a.O;
                cw[u][rb] = load_code_words<BITS>(rW, ok ? (uint32_t)o[rb] * a.w_row_bytes + (uint32_t)seg * (4u * BITS) : kOobOffset);
                sv[u][rb] = __int_as_float(buf_load4(rS, ok ? ((uint32_t)o[rb] * (uint32_t)a.G + j) * 4u : kOobOffset));
                if constexpr (FLOATZ) {
                    zv[u][rb] = __int_as_float(buf_load4(rZ, ok ? ((uint32_t)o[rb] * (uint32_t)a.G + j) * 4u : kOobOffset));
                } else {
                    const uint32_t wi = (j * BITS) >> 5;
                    zw0[u][rb] = (uint32_t)buf_load4(rZ, ok ? ((uint32_t)o[rb] * a.z_row_words + wi) * 4u : kOobOffset);
                    zw1[u][rb] = (BITS == 3) ? (uint32_t)buf_load4(rZ, ok ? ((uint32_t)o[rb] * a.z_row_words + wi + 1u) * 4u : kOobOffset) : 0u;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kGemvUnroll; ++u) {
            const int seg = (c0 + u) * 4 + kq;
            // token fragments: lane (n, kq) holds slots kq*8.. of MFMA t of segment seg.  A segment past the end of the row
            // (or of this wave's range) has s = 0, i.e. all-zero weights: any finite token data will do for it.
            const bf16_t *xrow = xlane + (seg < n_segs ? seg : 0) * 32;
            const bf16x8 b0 = *reinterpret_cast<const bf16x8 *>(xrow + 0);
            const bf16x8 b1 = *reinterpret_cast<const bf16x8 *>(xrow + 8);
            const bf16x8 b2 = *reinterpret_cast<const bf16x8 *>(xrow + 16);
            const bf16x8 b3 = *reinterpret_cast<const bf16x8 *>(xrow + 24);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                if constexpr (!FLOATZ) {
                    const uint32_t j = a.spg_magic ? __umulhi((uint32_t)seg, a.spg_magic) : (uint32_t)seg, sh = (j * BITS) & 31u;
                    const uint64_t two = (uint64_t)zw0[u][rb] | ((uint64_t)zw1[u][rb] << 32);
                    zv[u][rb] = (float)((uint32_t)(two >> sh) & ((1u << BITS) - 1u));
                }
                WhatTable<BITS> tab;
                tab.build(sv[u][rb], zv[u][rb]);
                acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(eight_of<BITS, 0>(tab, cw[u][rb]), b0, acc[rb], 0, 0, 0);
                acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(eight_of<BITS, 1>(tab, cw[u][rb]), b1, acc[rb], 0, 0, 0);
                acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(eight_of<BITS, 2>(tab, cw[u][rb]), b2, acc[rb], 0, 0, 0);
                acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(eight_of<BITS, 3>(tab, cw[u][rb]), b3, acc[rb], 0, 0, 0);
            }
        }
    }

    // ---- sum the four waves' partial tiles (wave order) and store ------------------------------------------
    __syncthreads();                                  // everyone is done reading xs
    // acc[i] = D[row 4*(lane/16) + i][col lane%16]: row = output row of the block, col = token
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int i = 0; i < 4; ++i) red[((wave * RB + rb) * 16 + 4 * kq + i) * 16 + r] = acc[rb][i];
    __syncthreads();
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row = tid >> 4, n = tid & 15;       // 256 threads = 16 rows x 16 tokens
        const int oo = (blockIdx.x * RB + rb) * kGemvRows + row;
        if (n < a.T && oo < a.O) {
            float v = 0.0f;
#pragma unroll
            for (int w = 0; w < kGemvWaves; ++w) v += red[((w * RB + rb) * 16 + row) * 16 + n];
            a.Y[(size_t)n * a.O + oo] = (bf16_t)v;
        }
    }
}

// The fast path.  A lane owns a RUN of 8 consecutive segments (256 inputs) of its row per trip: 16-byte loads of the
// codes, and the run's step sizes / zero points (NG = 8, 4, 2 or 1 groups per run, i.e. g = 32, 64, 128, or any multiple
// of 256) fetched with one or two wide loads instead of one small load per segment, which is what the memory path can
// sustain: per-segment 4-byte loads from 16 rows x 3 arrays thrash the 16 KB L1 and move ~7 bytes per useful byte.
// The value table is rebuilt only when the group changes.
// MW ("more waves"): launched with one wave per run of a row, 5 to 8 of them, instead of four waves that take turns.  For
// matrices with few row blocks (less than 16 waves per compute unit with four) that puts every load of the launch in
// flight at once (measured 4-7 % faster at 5120 x 5120, 13824 x 5120 and 8192 x 8192); with many row blocks the chip is
// full anyway and the fixed-size version, whose loops the compiler knows, is the faster one.
template <int BITS, bool FLOATZ, int NG, bool MW>
__global__ __launch_bounds__(64 * (MW ? kGemvMaxWaves : kGemvWaves)) void k_gemv_run(const GemvArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t *xs = reinterpret_cast<bf16_t *>(smem_raw);                       // [T][I], contraction-slot order
    float *red = reinterpret_cast<float *>(smem_raw);                        // reused after the loop: [waves][16][16]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_waves = MW ? (int)(blockDim.x >> 6) : kGemvWaves;
    const int r = lane & 15, kq = lane >> 4;
    const int n_segs = a.I >> 5;
    const int o = blockIdx.x * kGemvRows + r;
    const bool row_ok = o < a.O;

    const __amdgpu_buffer_rsrc_t rW = make_rsrc(a.Wp, a.w_bytes);
    const __amdgpu_buffer_rsrc_t rS = make_rsrc(a.s, a.s_bytes);
    const __amdgpu_buffer_rsrc_t rZ = make_rsrc(FLOATZ ? (const void *)a.zf : (const void *)a.zp, a.z_bytes);
    constexpr int CW = 2 * BITS;                      // 16-byte loads per run of 8 segments
    constexpr int SW = NG >= 4 ? NG / 4 : 1;          // 16-byte loads of step sizes (shorter loads for NG = 2, 1)

    auto load_run = [&](int sc, uintx4 (&cq)[CW], floatx4 (&sq)[SW], floatx4 (&zq)[SW], uint32_t (&zw)[2]) {
        const int seg0 = sc * 32 + kq * 8;
        const bool ok = row_ok && seg0 < n_segs;
        const uint32_t base = (uint32_t)o * a.w_row_bytes + (uint32_t)seg0 * (4u * BITS);
#pragma unroll
        for (int q = 0; q < CW; ++q) {
            const intx4 v = buf_load16(rW, ok ? base + 16u * q : kOobOffset);
            cq[q] = uintx4{(uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2], (uint32_t)v[3]};
        }
        // first group of the run: runs are 256 inputs, groups NG per run (NG > 1) or a whole number of runs per group
        const uint32_t j0 = NG > 1 ? (uint32_t)(seg0 >> 3) * NG : (a.spg_magic ? __umulhi((uint32_t)seg0, a.spg_magic) : (uint32_t)seg0);
        const uint32_t gi = ok ? ((uint32_t)o * (uint32_t)a.G + j0) * 4u : kOobOffset;
        auto wide = [&](__amdgpu_buffer_rsrc_t rr, floatx4 (&dst)[SW]) {
            if constexpr (NG >= 4) {
#pragma unroll
                for (int q = 0; q < SW; ++q) {
                    const intx4 v = buf_load16(rr, ok ? gi + 16u * q : kOobOffset);
                    dst[q] = floatx4{__int_as_float(v[0]), __int_as_float(v[1]), __int_as_float(v[2]), __int_as_float(v[3])};
                }
            } else if constexpr (NG == 2) {
                const intx2 v = buf_load8(rr, gi);
                dst[0] = floatx4{__int_as_float(v[0]), __int_as_float(v[1]), 0.0f, 0.0f};
            } else {
                dst[0] = floatx4{__int_as_float(buf_load4(rr, gi)), 0.0f, 0.0f, 0.0f};
            }
        };
        wide(rS, sq);
        if constexpr (FLOATZ) {
            wide(rZ, zq);
        } else {
            const uint32_t wi = (j0 * BITS) >> 5;
            zw[0] = (uint32_t)buf_load4(rZ, ok ? ((uint32_t)o * a.z_row_words + wi) * 4u : kOobOffset);
            zw[1] = (BITS == 3) ? (uint32_t)buf_load4(rZ, ok ? ((uint32_t)o * a.z_row_words + wi + 1u) * 4u : kOobOffset) : 0u;
        }
    };

    const int n_runs = (n_segs + 31) / 32;            // trips of one wave cover 32 segments (4 lane groups x 8)

    // ---- stage the token rows in slot order (one 32-input segment per thread and trip) ---------------------
    for (int e = tid; e < a.T * n_segs; e += 64 * n_waves) {
        const int n = e / n_segs, seg = e - n * n_segs;
        const bf16_t *src = a.X + (size_t)n * a.I + seg * 32;
        bf16_t *dst = xs + (size_t)n * a.I + seg * 32;
        bf16x8 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const bf16x8 *>(src + 8 * q);
#pragma unroll
        for (int c = 0; c < 32; ++c) dst[code_slot<BITS>(c)] = v[c / 8][c % 8];
    }
    __syncthreads();

    const bf16_t *xlane = xs + (size_t)((lane & 15) < a.T ? (lane & 15) : 0) * a.I;
    floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int sc = wave; sc < n_runs; sc += n_waves) {
        const int seg0 = sc * 32 + kq * 8;
        uintx4 cq[CW];
        floatx4 sq[SW], zq[SW];
        uint32_t zw[2] = {0u, 0u};
        load_run(sc, cq, sq, zq, zw);
        WhatTable<BITS> tab;
        const uint32_t j0 = NG > 1 ? (uint32_t)(seg0 >> 3) * NG : (a.spg_magic ? __umulhi((uint32_t)seg0, a.spg_magic) : (uint32_t)seg0);
        const uint64_t zbits = ((uint64_t)zw[0] | ((uint64_t)zw[1] << 32)) >> ((j0 * BITS) & 31u);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            constexpr int kSegsPerGroup = 8 / NG;
            const bool seg_ok = seg0 + u < n_segs;
            if (u % kSegsPerGroup == 0) {
                const int gsel = u / kSegsPerGroup;                                   // compile time after unrolling
                const float sv = sq[gsel / 4][gsel % 4];
                const float zv = FLOATZ ? zq[gsel / 4][gsel % 4] : (float)((uint32_t)(zbits >> (gsel * BITS)) & ((1u << BITS) - 1u));
                // a segment past the end of the row shares its loads with the next row: its weights are forced to zero
                tab.build(seg_ok ? sv : 0.0f, zv);
            }
            CodeWords<BITS> cw;
#pragma unroll
            for (int k = 0; k < BITS; ++k) cw.w[k] = cq[(u * BITS + k) / 4][(u * BITS + k) % 4];
            const bf16_t *xrow = xlane + (seg_ok ? seg0 + u : 0) * 32;
            const bf16x8 b0 = *reinterpret_cast<const bf16x8 *>(xrow + 0);
            const bf16x8 b1 = *reinterpret_cast<const bf16x8 *>(xrow + 8);
            const bf16x8 b2 = *reinterpret_cast<const bf16x8 *>(xrow + 16);
            const bf16x8 b3 = *reinterpret_cast<const bf16x8 *>(xrow + 24);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(eight_of<BITS, 0>(tab, cw), b0, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(eight_of<BITS, 1>(tab, cw), b1, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(eight_of<BITS, 2>(tab, cw), b2, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(eight_of<BITS, 3>(tab, cw), b3, acc, 0, 0, 0);
        }
    }

    // ---- sum the waves' partial tiles (wave order) and store ------------------------------------------
    __syncthreads();                                  // everyone is done reading xs
#pragma unroll
    for (int i = 0; i < 4; ++i) red[(wave * 16 + 4 * kq + i) * 16 + r] = acc[i];
    __syncthreads();
    if (!MW || tid < 256) {
        const int row = tid >> 4, n = tid & 15;       // 256 threads = 16 rows x 16 tokens
        const int oo = blockIdx.x * kGemvRows + row;
        if (n < a.T && oo < a.O) {
            float v = 0.0f;
#pragma unroll 4
            for (int w = 0; w < n_waves; ++w) v += red[(w * 16 + row) * 16 + n];
            a.Y[(size_t)n * a.O + oo] = (bf16_t)v;
        }
    }
}

}  // namespace

bool gemv_applies(const Problem &p)
{
    return p.act_bf16 && p.T >= 1 && p.T <= 16 && (size_t)p.T * p.I * 2 <= 64 * 1024;
}

void launch_gemv(const Problem &p, const void *X, const void *Wpacked, const float *s, const void *zpacked,
                 const float *zfloat, void *Y, hipStream_t st)
{
    GemvArgs a{};
    a.X = (const bf16_t *)X; a.Wp = (const uint32_t *)Wpacked; a.s = s; a.zp = (const uint32_t *)zpacked; a.zf = zfloat;
    a.Y = (bf16_t *)Y;
    a.T = (int)p.T; a.I = (int)p.I; a.O = (int)p.O; a.G = (int)p.G; a.g = (int)p.g;
    a.spg_magic = (p.g == 32) ? 0u : (uint32_t)((((uint64_t)1 << 32) + (uint64_t)(p.g / 32) - 1) / (uint64_t)(p.g / 32));
    a.w_row_bytes = (uint32_t)(p.I * p.bits / 8);
    a.z_row_words = (uint32_t)((p.G * p.bits + 31) / 32);
    a.w_bytes = (uint32_t)(p.O * p.I * p.bits / 8);
    a.s_bytes = (uint32_t)(p.O * p.G * 4);
    a.z_bytes = zfloat != nullptr ? a.s_bytes : (uint32_t)(p.O * a.z_row_words * 4);
    // groups per run of 256 inputs; 0 = a group size the run kernel does not take
    const int ng = p.g == 32 ? 8 : p.g == 64 ? 4 : p.g == 128 ? 2 : (p.g % 256 == 0 ? 1 : 0);
    // a wave per run of 1024 inputs when four waves per row block would leave the chip short of waves (see k_gemv_run)
    const int n_blocks = (int)((p.O + kGemvRows - 1) / kGemvRows), n_runs = (int)((p.I / 32 + 31) / 32);
    const bool more_waves = ng != 0 && n_runs > kGemvWaves && n_blocks * kGemvWaves < 16 * 256;
    const int waves = more_waves ? std::min(n_runs, kGemvMaxWaves) : kGemvWaves;
    const size_t red_bytes = (size_t)waves * 16 * 16 * 4;
    const size_t smem = (size_t)p.T * p.I * 2 > red_bytes ? (size_t)p.T * p.I * 2 : red_bytes;
    const dim3 grid((unsigned)n_blocks), block(64 * waves);
    if (ng == 1) {          // magic for "group of segment": exact for segment * (g/32) < 2^32
        a.spg_magic = (uint32_t)((((uint64_t)1 << 32) + (uint64_t)(p.g / 32) - 1) / (uint64_t)(p.g / 32));
    }
#define EQAT_GEMV_NG(B, FZ, MW)                                                                   \
    do {                                                                                          \
        if (ng == 8) k_gemv_run<B, FZ, 8, MW><<<grid, block, smem, st>>>(a);                       \
        else if (ng == 4) k_gemv_run<B, FZ, 4, MW><<<grid, block, smem, st>>>(a);                  \
        else if (ng == 2) k_gemv_run<B, FZ, 2, MW><<<grid, block, smem, st>>>(a);                  \
        else k_gemv_run<B, FZ, 1, MW><<<grid, block, smem, st>>>(a);                               \
    } while (0)
#define EQAT_GEMV_RUN(B, FZ)                                                                      \
    do {                                                                                          \
        if (ng == 0) k_gemv_any<B, FZ, 1><<<grid, block, smem, st>>>(a);                           \
        else if (more_waves) EQAT_GEMV_NG(B, FZ, true);                                           \
        else EQAT_GEMV_NG(B, FZ, false);                                                          \
    } while (0)
#define EQAT_GEMV(B) do { if (zfloat != nullptr) EQAT_GEMV_RUN(B, true); else EQAT_GEMV_RUN(B, false); } while (0)
    if (p.bits == 2) EQAT_GEMV(2); else if (p.bits == 3) EQAT_GEMV(3); else EQAT_GEMV(4);
#undef EQAT_GEMV_RUN
#undef EQAT_GEMV_NG
#undef EQAT_GEMV
}

}  // namespace eqat
