// HBM-bound passes: min/max initialisation, the quantize pass (Eq.(1) -> packed N-bit codes),
// zero-point packing / unpacking, code unpacking, and the small reductions the GEMM epilogues need.
#include "common.h"
#include "kernels.h"

namespace eqat {

// ---------------------------------------------------------------------------------------------
// Eq.(1) for one weight.  The code must equal clamp(round_half_even(fl32(w/s)) + zbar, 0, Qmax) exactly.  The exact
// quotient costs a dozen instructions, so k_quantize first uses w * (1/s), which is within 2^-22 relative of it; only
// a chunk in which some product lies too close to a rounding tie - where the cheap and the exact quotient could round
// differently - is redone with this exact division.
__device__ __forceinline__ float quant_exact(float w, float s) { return __builtin_rintf(w / s); }

template <typename WT> struct Chunk8;   // 8 consecutive weights of one lane
template <> struct Chunk8<bf16_t> {
    static constexpr int kBytes = 16;
    uintx4 v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const uintx4 *>(p); }
    __device__ __forceinline__ float get(int k) const
    {
        const uint32_t u = v[k >> 1];
        return __uint_as_float((k & 1) ? (u & 0xFFFF0000u) : (u << 16));
    }
};
template <> struct Chunk8<float> {
    static constexpr int kBytes = 32;
    floatx4 a, b;
    __device__ __forceinline__ void load(const float *p)
    {
        a = *reinterpret_cast<const floatx4 *>(p);
        b = *reinterpret_cast<const floatx4 *>(p + 4);
    }
    __device__ __forceinline__ float get(int k) const { return k < 4 ? a[k] : b[k - 4]; }
};

__device__ __forceinline__ uint32_t quad_bcast(uint32_t v, int k)
{
    // value of lane (lane & ~3) + k, through a DPP quad permute
    switch (k) {
    case 0: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x00, 0xF, 0xF, false);
    case 1: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x55, 0xF, 0xF, false);
    case 2: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xAA, 0xF, 0xF, false);
    default: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xFF, 0xF, 0xF, false);
    }
}

// The quantize pass.  One lane owns 8 consecutive weights (a 16- or 32-byte load); the four lanes of a
// quad own one 32-code segment, i.e. BITS output words, assembled with quad permutes.
//   codes     [O, I*BITS/32] words      packed stream (same layout as eqat_pack's Wpacked)
//   clampbits [O, I/8] bytes (CLAMPBITS) bit k of byte e/8: weight e was clamped by Eq.(1)
//   sz        [O, G] float2 or NULL     (s, zbar) per group, zbar = clamp(round(z), 0, Qmax)
// Rows are contiguous and g divides I, so weight e belongs to group e / g of the flattened [O*G] arrays.
// Per weight the common path costs: widen, multiply, round, two ops of tie test, clamp, convert, shift-add.
// The clamp is applied to round(w/s) against [-zbar, Qmax - zbar] and zbar is added once, as an integer, to
// all eight packed fields (the per-field sums stay inside [0, Qmax], so no carry crosses a field).
// WORK = false: the dense stream of the C ABI (eqat_pack).  WORK = true: the library's working layout (WorkCodes).
// Zero points at N bits: one thread per output word (tail bits of a row are zero).
template <int BITS>
__device__ __forceinline__ void pack_z_word(const float *__restrict__ z, uint32_t *__restrict__ zpacked, uint32_t t,
                                            uint32_t G, uint32_t row_words)
{
    const uint32_t row = t / row_words, w = t - row * row_words;
    constexpr float qmax = (float)((1 << BITS) - 1);
    const uint32_t bit0 = w * 32u;
    uint32_t j = bit0 / BITS;                   // first code with bits in this word
    uint64_t acc = 0;
    for (; j < G && j * BITS < bit0 + 32u; ++j) {
        const uint32_t code = (uint32_t)zbar_of(z[row * G + j], qmax);
        const int sh = (int)(j * BITS) - (int)bit0;         // may be negative for a code straddling in from the left
        acc |= sh >= 0 ? ((uint64_t)code << sh) : ((uint64_t)code >> (-sh));
    }
    zpacked[t] = (uint32_t)acc;
}

struct QuantizeArgs {
    const void *W; const float *s, *z;
    uint32_t *codes; uint8_t *clampbits; floatx2 *sz;
    uint32_t n_chunks, g; int g_shift;
    // eqat_pack only: the blocks past n_quant_blocks pack the zero points (one thread per word)
    uint32_t *zpacked; uint32_t n_quant_blocks, n_zwords, G, row_words;
    // words the launch clears on the side (arrival counters of the GEMM launches that follow); NULL: none
    uint32_t *zero_words; uint32_t n_zero;
};

// block / nblocks: this workgroup's number among those that share the job
__device__ __forceinline__ void clear_words(uint32_t *__restrict__ w, uint32_t n, uint32_t block, uint32_t nblocks)
{
    for (uint32_t i = block * blockDim.x + threadIdx.x; i < n; i += nblocks * blockDim.x) w[i] = 0u;
}

// Up to kMaxBatch matrices in one launch (the linears of a decoder block are 34-90 MB each at 7B size: alone, each would
// be a 10-25 us launch that spends a good part of its time filling and draining the chip).  Workgroups
// [first[i], first[i + 1]) work on matrix i.
struct QuantizeBatch { QuantizeArgs a[kMaxBatch]; uint32_t first[kMaxBatch + 1]; };
__device__ __forceinline__ int batch_slot(const uint32_t (&first)[kMaxBatch + 1], uint32_t block)
{
    int i = 0;
#pragma unroll
    for (int k = 1; k < kMaxBatch; ++k) i += block >= first[k] ? 1 : 0;      // first[k] of unused slots: the grid size
    return i;
}

constexpr int kQuantUnroll = 4;     // chunks per thread: 64 B (bf16) / 128 B (fp32) of W in flight per lane
// eqat_pack of one large bf16 matrix (the 70B-sized ones, 235 M weights): twice the loads in flight measured +5 %; on
// smaller matrices, with several matrices per launch and in the working-layout instantiations it measured 2-10 % slower.
constexpr int kPackUnrollLarge = 8;
constexpr size_t kPackLargeChunks = (size_t)1 << 24;     // 8-weight chunks: 134 M weights

template <typename WT, int BITS, bool CLAMPBITS, bool WORK, int U = kQuantUnroll>
__global__ __launch_bounds__(256) void k_quantize(const QuantizeBatch batch)
{
    const int slot = batch_slot(batch.first, blockIdx.x);
    const QuantizeArgs &a = batch.a[slot];
    const uint32_t block = blockIdx.x - batch.first[slot];
    if (a.zero_words != nullptr) clear_words(a.zero_words, a.n_zero, block, batch.first[slot + 1] - batch.first[slot]);
    if (block >= a.n_quant_blocks) {
        const uint32_t t = (block - a.n_quant_blocks) * 256u + threadIdx.x;
        if (t < a.n_zwords) pack_z_word<BITS>(a.z, a.zpacked, t, a.G, a.row_words);
        return;
    }
    const WT *__restrict__ W = reinterpret_cast<const WT *>(a.W);
    constexpr float qmax = (float)((1 << BITS) - 1);
    const uint32_t c0 = block * (256u * U) + threadIdx.x;   // chunk index; n_chunks % 4 == 0 so quads stay whole
    // all loads of the thread's U chunks first: the pass lives on bytes in flight
    Chunk8<WT> ch[U];
    uint32_t gi[U];
    float sv[U], zb[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t c = c0 + u * 256u;
        const uint32_t cc = c < a.n_chunks ? c : 0u;             // past the end: recompute chunk 0, store nothing
        const uint32_t e = cc * 8u;
        gi[u] = a.g_shift >= 0 ? (e >> a.g_shift) : (e / a.g);
        ch[u].load(W + e);
        sv[u] = a.s[gi[u]];
        zb[u] = a.z[gi[u]];
    }
    const uint32_t q4 = threadIdx.x & 3u;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t c = c0 + u * 256u;
        if (c >= a.n_chunks) break;
        const uint32_t e = c * 8u;
        const float zbar = zbar_of(zb[u], qmax);
        if (a.sz != nullptr && e == gi[u] * a.g) { floatx2 o; o[0] = sv[u]; o[1] = zbar; a.sz[gi[u]] = o; }
        const float rinv = __builtin_amdgcn_rcpf(sv[u]);          // 1 ulp; s is a normal number
        const float lo = -zbar, hi = qmax - zbar;
        // Far from a rounding tie the cheap quotient w * rcp(s) (within 2^-22 relative of w/s) rounds like the exact one.
        // Only weights whose code is not clamped matter, and for those |w/s| <= |zbar| + Qmax + 1.
        const float thr = 0.5f - 0x1p-20f * (__builtin_fabsf(zbar) + qmax + 2.0f);
        float r[8];
        float worst = 0.0f;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float t = ch[u].get(k) * rinv;
            r[k] = __builtin_rintf(t);
            worst = __builtin_fmaxf(worst, __builtin_fabsf(t - r[k]));
        }
        if (worst >= thr) {
#pragma unroll
            for (int k = 0; k < 8; ++k) r[k] = quant_exact(ch[u].get(k), sv[u]);
        }
        uint32_t p = 0, cb = 0;
        if constexpr (!WORK) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float qc = __builtin_amdgcn_fmed3f(r[k], lo, hi);      // lo <= hi: the median is the clamp
                p += (uint32_t)(int)qc << (k * BITS);          // two's complement: fields may be negative until zbar is added
                if (CLAMPBITS) cb |= (qc != r[k] ? 1u : 0u) << k;
            }
            constexpr uint32_t ones = BITS == 2 ? 0x5555u : BITS == 3 ? 0x249249u : 0x11111111u;   // a one in every field
            p += (uint32_t)(int)zbar * ones;
            if (CLAMPBITS) a.clampbits[c] = (uint8_t)cb;

            const uint32_t pu = p & (BITS == 4 ? 0xFFFFFFFFu : ((1u << (8 * BITS)) - 1u));
            const uint32_t p0 = quad_bcast(pu, 0), p1 = quad_bcast(pu, 1), p2 = quad_bcast(pu, 2), p3 = quad_bcast(pu, 3);
            uint32_t word;
            if constexpr (BITS == 2) {
                word = (q4 == 0) ? (p0 | (p1 << 16)) : (p2 | (p3 << 16));
            } else if constexpr (BITS == 3) {
                word = (q4 == 0) ? (p0 | (p1 << 24)) : (q4 == 1) ? ((p1 >> 8) | (p2 << 16)) : ((p2 >> 16) | (p3 << 8));
            } else {
                word = (q4 == 0) ? p0 : (q4 == 1) ? p1 : (q4 == 2) ? p2 : p3;
            }
            if (q4 < (uint32_t)BITS) a.codes[(c >> 2) * BITS + q4] = word;
        } else {
            // working layout: this lane's code k goes to byte k % 4, field k / 4 (+ 2 fields for the odd lane of a 2-bit pair)
            constexpr int F = WorkCodes<BITS>::kField;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float qc = __builtin_amdgcn_fmed3f(r[k], lo, hi);
                p += (uint32_t)(int)qc << (8 * (k % 4) + F * (k / 4));
                if (CLAMPBITS) cb |= (qc != r[k] ? 1u : 0u) << k;
            }
            constexpr uint32_t ones = BITS == 2 ? 0x05050505u : 0x11111111u;
            p += (uint32_t)(int)zbar * ones;
            if (CLAMPBITS) a.clampbits[c] = (uint8_t)cb;
            if constexpr (BITS == 2) {
                const uint32_t mine = p & 0x0F0F0F0Fu;
                const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mine, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
                if ((q4 & 1u) == 0) a.codes[(c >> 2) * 2 + (q4 >> 1)] = mine | (other << 4);
            } else {
                a.codes[c] = p & WorkCodes<BITS>::kByteMask * 0x11u;
            }
        }
    }
}

// The dense stream of the C ABI -> the working layout (one thread per 32-code segment).
template <int BITS>
__device__ __forceinline__ void repack_segment(const uint32_t *__restrict__ packed, uint32_t *__restrict__ work, uint32_t t)
{
    uint32_t in[BITS];
#pragma unroll
    for (int k = 0; k < BITS; ++k) in[k] = packed[(size_t)t * BITS + k];
    uint32_t out[WorkCodes<BITS>::kWords] = {};
#pragma unroll
    for (int e = 0; e < 32; ++e)
        out[WorkCodes<BITS>::word_of(e)] |= code_at_rt<BITS>(in, e) << WorkCodes<BITS>::bit_of(e);
#pragma unroll
    for (int k = 0; k < WorkCodes<BITS>::kWords; ++k) work[(size_t)t * WorkCodes<BITS>::kWords + k] = out[k];
}

// (s, z) pair of group t for the E2E-QP kernels: z from the packed N-bit zero points, or from a float array.
// zb_out (may be NULL) also receives the zero point alone; sz may be NULL when only that is wanted.
template <int BITS>
__device__ __forceinline__ void pair_sz(const float *__restrict__ s, const uint32_t *__restrict__ zpacked,
                                        const float *__restrict__ zfloat, floatx2 *__restrict__ sz, float *__restrict__ zb_out,
                                        uint32_t t, uint32_t G, uint32_t row_words)
{
    float zv;
    if (zfloat != nullptr) {
        zv = zfloat[t];
    } else {
        const uint32_t row = t / G, j = t - row * G;
        const uint32_t bit = j * BITS, wi = bit >> 5, sh = bit & 31u;
        uint64_t two = zpacked[row * row_words + wi];
        if (sh + BITS > 32u) two |= (uint64_t)zpacked[row * row_words + wi + 1] << 32;
        zv = (float)((uint32_t)(two >> sh) & ((1u << BITS) - 1u));
    }
    if (zb_out != nullptr) zb_out[t] = zv;
    if (sz != nullptr) { floatx2 o; o[0] = s[t]; o[1] = zv; sz[t] = o; }
}

// What an E2E-QP call needs before its GEMMs, in one launch: the first n_repack_blocks workgroups re-lay the codes from
// the dense stream into the working layout (packed == NULL: none; a prepared layer has them already), the rest write the
// (s, z) pairs (and / or the zero points alone: what eqat_qlinear_prepare keeps).
template <int BITS>
__global__ __launch_bounds__(256) void k_e2e_prepare(const uint32_t *__restrict__ packed, uint32_t *__restrict__ work,
                                                     uint32_t n_segs, uint32_t n_repack_blocks,
                                                     const float *__restrict__ s, const uint32_t *__restrict__ zpacked,
                                                     const float *__restrict__ zfloat, floatx2 *__restrict__ sz,
                                                     float *__restrict__ zb_out, uint32_t n_groups, uint32_t G,
                                                     uint32_t row_words, uint32_t *__restrict__ zero_words, uint32_t n_zero)
{
    if (zero_words != nullptr) clear_words(zero_words, n_zero, blockIdx.x, gridDim.x);
    if (blockIdx.x < n_repack_blocks) {
        const uint32_t t = blockIdx.x * 256u + threadIdx.x;
        if (t < n_segs) repack_segment<BITS>(packed, work, t);
    } else {
        const uint32_t t = (blockIdx.x - n_repack_blocks) * 256u + threadIdx.x;
        if (t < n_groups) pair_sz<BITS>(s, zpacked, zfloat, sz, zb_out, t, G, row_words);
    }
}

template <int BITS>
__global__ __launch_bounds__(256) void k_unpack_codes(const uint32_t *__restrict__ packed, int32_t *__restrict__ out,
                                                      uint32_t n_segs)
{
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    if (t >= n_segs) return;
    uint32_t w[BITS];
#pragma unroll
    for (int k = 0; k < BITS; ++k) w[k] = packed[(size_t)t * BITS + k];
    for (int k = 0; k < 32; ++k) out[(size_t)t * 32 + k] = (int32_t)code_at_rt<BITS>(w, k);
}
template <int BITS>
__global__ __launch_bounds__(256) void k_unpack_z(const uint32_t *__restrict__ zpacked, int32_t *__restrict__ out,
                                                  uint32_t O, uint32_t G, uint32_t row_words)
{
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    if (t >= O * G) return;
    const uint32_t row = t / G, j = t - row * G;
    const uint32_t bit = j * BITS, wi = bit >> 5, sh = bit & 31u;
    uint64_t two = zpacked[row * row_words + wi];
    if (sh + BITS > 32u) two |= (uint64_t)zpacked[row * row_words + wi + 1] << 32;
    out[t] = (int32_t)((uint32_t)(two >> sh) & ((1u << BITS) - 1u));
}

// Test aid: one thread per 32-code segment of the working layout; the first n_groups threads also split the
// (s, zero point) pairs.
template <int BITS>
__global__ __launch_bounds__(256) void k_unpack_work(const uint32_t *__restrict__ work, const uint32_t *__restrict__ clampbits,
                                                     const floatx2 *__restrict__ sz, int32_t *__restrict__ codes,
                                                     uint8_t *__restrict__ clamped, float *__restrict__ zbar, uint32_t n_segs,
                                                     uint32_t n_groups)
{
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    if (zbar != nullptr && t < n_groups) zbar[t] = sz[t][1];
    if (t >= n_segs) return;
    typedef WorkCodes<BITS> WC;
    if (codes != nullptr) {
        uint32_t w[WC::kWords];
#pragma unroll
        for (int k = 0; k < WC::kWords; ++k) w[k] = work[(size_t)t * WC::kWords + k];
#pragma unroll
        for (int e = 0; e < 32; ++e)
            codes[(size_t)t * 32 + e] = (int32_t)((w[WC::word_of(e)] >> WC::bit_of(e)) & ((1u << BITS) - 1u));
    }
    if (clamped != nullptr) {
        const uint32_t bits = clampbits[t];                 // bit e of the segment's word: weight e was clamped
        for (int e = 0; e < 32; ++e) clamped[(size_t)t * 32 + e] = (uint8_t)((bits >> e) & 1u);
    }
}

// ---------------------------------------------------------------------------------------------
// min/max initialisation.  LPG = lanes per group (g/8), a power of two <= 64: one lane reduces its 8
// weights, an xor butterfly reduces the group.
struct InitBatch {
    const void *W[kMaxBatch]; float *s[kMaxBatch], *z[kMaxBatch];
    uint32_t n[kMaxBatch];                 // chunks of 8 weights (small kernel) / groups (wave kernel)
    uint32_t g[kMaxBatch];                 // group size (wave kernel)
    uint32_t first[kMaxBatch + 1];
};

template <typename WT, int LPG>
__global__ __launch_bounds__(256) void k_init_minmax_small(const InitBatch b, float qmax)
{
    constexpr int U = kQuantUnroll;
    const int slot = batch_slot(b.first, blockIdx.x);
    const WT *__restrict__ W = reinterpret_cast<const WT *>(b.W[slot]);
    float *__restrict__ s = b.s[slot], *__restrict__ z = b.z[slot];
    const uint32_t n_chunks = b.n[slot];
    const uint32_t c0 = (blockIdx.x - b.first[slot]) * (256u * U) + threadIdx.x;
    // n_chunks % LPG == 0 and 256 % LPG == 0: a group never straddles the end of the array or of a 256-chunk slice
    Chunk8<WT> ch[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t c = c0 + u * 256u;
        ch[u].load(W + (size_t)(c < n_chunks ? c : 0u) * 8);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t c = c0 + u * 256u;
        if (c >= n_chunks) break;
        float lo = ch[u].get(0), hi = lo;
#pragma unroll
        for (int k = 1; k < 8; ++k) { lo = __builtin_fminf(lo, ch[u].get(k)); hi = __builtin_fmaxf(hi, ch[u].get(k)); }
#pragma unroll
        for (int m = 1; m < LPG; m <<= 1) {
            lo = __builtin_fminf(lo, __shfl_xor(lo, m));
            hi = __builtin_fmaxf(hi, __shfl_xor(hi, m));
        }
        if ((c & (LPG - 1)) == 0) {
            float step = (hi - lo) / qmax;
            if (!(step >= 1e-10f)) step = 1e-10f;
            float zf = __builtin_rintf((-lo) / step);
            zf = __builtin_fminf(__builtin_fmaxf(zf, 0.0f), qmax);
            s[c / LPG] = step;
            z[c / LPG] = zf;
        }
    }
}
// Any other group size: one wavefront per group.
template <typename WT>
__global__ __launch_bounds__(256) void k_init_minmax_wave(const InitBatch b, float qmax)
{
    const int slot = batch_slot(b.first, blockIdx.x);
    const WT *__restrict__ W = reinterpret_cast<const WT *>(b.W[slot]);
    float *__restrict__ s = b.s[slot], *__restrict__ z = b.z[slot];
    const uint32_t n_groups = b.n[slot], g = b.g[slot];
    const uint32_t grp = (blockIdx.x - b.first[slot]) * 4u + (threadIdx.x >> 6);
    if (grp >= n_groups) return;
    const uint32_t lane = threadIdx.x & 63u;
    const WT *base = W + (size_t)grp * g;
    float lo = __builtin_inff(), hi = -__builtin_inff();
    for (uint32_t c = lane; c < g / 8u; c += 64u) {
        Chunk8<WT> ch;
        ch.load(base + c * 8u);
#pragma unroll
        for (int k = 0; k < 8; ++k) { lo = __builtin_fminf(lo, ch.get(k)); hi = __builtin_fmaxf(hi, ch.get(k)); }
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        lo = __builtin_fminf(lo, __shfl_xor(lo, m));
        hi = __builtin_fmaxf(hi, __shfl_xor(hi, m));
    }
    if (lane == 0) {
        float step = (hi - lo) / qmax;
        if (!(step >= 1e-10f)) step = 1e-10f;
        float zf = __builtin_rintf((-lo) / step);
        zf = __builtin_fminf(__builtin_fmaxf(zf, 0.0f), qmax);
        s[grp] = step;
        z[grp] = zf;
    }
}

// out[o,j] = sum of the n_per consecutive per-32-column partials of group j, in index order;
// `scale_by_s` multiplies by -s[o,j] (turns a sum of clamped dWhat into dz).
__global__ __launch_bounds__(256) void k_reduce_partials(const float *__restrict__ part, float *__restrict__ out,
                                                         const float *__restrict__ s, uint32_t n_out, uint32_t n_per,
                                                         int scale_by_s)
{
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    if (t >= n_out) return;
    float acc = 0.0f;
    for (uint32_t k = 0; k < n_per; ++k) acc += part[(size_t)t * n_per + k];
    out[t] = scale_by_s ? -s[t] * acc : acc;
}

// ---------------------------------------------------------------------------------------------
// host-side launchers

static inline unsigned blocks_for(size_t n, unsigned per = 256) { return (unsigned)((n + per - 1) / per); }

static inline int pow2_shift(int64_t v)
{
    for (int k = 0; k < 31; ++k) if (((int64_t)1 << k) == v) return k;
    return -1;
}

static QuantizeArgs quantize_args(const QuantizeJob &j, int unroll)
{
    const Problem &p = j.p;
    QuantizeArgs a{};
    a.zero_words = j.zero_words; a.n_zero = j.n_zero;
    a.W = j.W; a.s = j.s; a.z = j.z; a.codes = (uint32_t *)j.codes; a.clampbits = (uint8_t *)j.clampbits; a.sz = (floatx2 *)j.sz;
    a.n_chunks = (uint32_t)((size_t)p.O * p.I / 8); a.g = (uint32_t)p.g; a.g_shift = pow2_shift(p.g);
    a.n_quant_blocks = blocks_for(a.n_chunks, 256 * unroll);
    a.zpacked = (uint32_t *)j.zpacked; a.G = (uint32_t)p.G; a.row_words = (uint32_t)((p.G * p.bits + 31) / 32);
    a.n_zwords = j.zpacked != nullptr ? (uint32_t)p.O * a.row_words : 0u;
    return a;
}

template <typename WT, int BITS>
static void quantize_t(const QuantizeJob *jobs, int n, bool for_pack, hipStream_t st)
{
    QuantizeBatch b{};
    uint32_t first = 0;
    const bool large_pack = for_pack && n == 1 && sizeof(WT) == 2 && (size_t)jobs[0].p.O * jobs[0].p.I / 8 >= kPackLargeChunks;
    for (int i = 0; i < n; ++i) {
        b.a[i] = quantize_args(jobs[i], large_pack ? kPackUnrollLarge : kQuantUnroll);
        b.first[i] = first;
        first += b.a[i].n_quant_blocks + blocks_for(b.a[i].n_zwords);
    }
    for (int i = n; i <= kMaxBatch; ++i) b.first[i] = first;
    const dim3 grid(first), block(256);
    // eqat_pack: dense stream, no clamp plane;
    // the quantize pass of the Block-AP calls: working layout, clamp plane for the backward
    if constexpr (sizeof(WT) == 2) {
        if (large_pack) { k_quantize<WT, BITS, false, false, kPackUnrollLarge><<<grid, block, 0, st>>>(b); return; }
    }
    if (for_pack) k_quantize<WT, BITS, false, false><<<grid, block, 0, st>>>(b);
    else if (jobs[0].clampbits != nullptr) k_quantize<WT, BITS, true, true><<<grid, block, 0, st>>>(b);
    else k_quantize<WT, BITS, false, true><<<grid, block, 0, st>>>(b);
}

void launch_quantize_batch(const QuantizeJob *jobs, int n, bool for_pack, hipStream_t st)
{
    const Problem &p = jobs[0].p;        // all jobs share bits, weight dtype and whether a clamp plane is written
#define EQAT_Q(WT, B) quantize_t<WT, B>(jobs, n, for_pack, st)
    if (p.w_bf16) { if (p.bits == 2) EQAT_Q(bf16_t, 2); else if (p.bits == 3) EQAT_Q(bf16_t, 3); else EQAT_Q(bf16_t, 4); }
    else          { if (p.bits == 2) EQAT_Q(float, 2);  else if (p.bits == 3) EQAT_Q(float, 3);  else EQAT_Q(float, 4); }
#undef EQAT_Q
}

void launch_quantize(const Problem &p, const void *W, const float *s, const float *z, void *codes, void *clampbits,
                     void *sz, void *zpacked, bool for_pack, uint32_t *zero_words, uint32_t n_zero, hipStream_t st)
{
    const QuantizeJob j{p, W, s, z, codes, clampbits, sz, zpacked, zero_words, n_zero};
    launch_quantize_batch(&j, 1, for_pack, st);
}

void launch_e2e_prepare(const Problem &p, const void *packed, void *work, const float *s, const void *zpacked,
                        const float *zfloat, void *sz, float *zb_out, uint32_t *zero_words, uint32_t n_zero, hipStream_t st)
{
    const uint32_t n_segs = packed != nullptr ? (uint32_t)((size_t)p.O * p.I / 32) : 0u;
    const uint32_t nb = blocks_for(n_segs), n_groups = (uint32_t)((size_t)p.O * p.G);
    const uint32_t row_words = (uint32_t)((p.G * p.bits + 31) / 32);
    const dim3 grid(nb + blocks_for(n_groups)), block(256);
#define EQAT_PREP(B) k_e2e_prepare<B><<<grid, block, 0, st>>>((const uint32_t *)packed, (uint32_t *)work, n_segs, nb, s, \
                                                             (const uint32_t *)zpacked, zfloat, (floatx2 *)sz, zb_out, \
                                                             n_groups, (uint32_t)p.G, row_words, zero_words, n_zero)
    if (p.bits == 2) EQAT_PREP(2); else if (p.bits == 3) EQAT_PREP(3); else EQAT_PREP(4);
#undef EQAT_PREP
}

void launch_unpack(const Problem &p, const void *Wpacked, const void *zpacked, int32_t *codes, int32_t *zcodes, hipStream_t st)
{
    const uint32_t row_words = (uint32_t)((p.G * p.bits + 31) / 32);
    if (codes != nullptr) {
        const uint32_t n_segs = (uint32_t)((size_t)p.O * p.I / 32);
        const dim3 grid(blocks_for(n_segs)), block(256);
        if (p.bits == 2) k_unpack_codes<2><<<grid, block, 0, st>>>((const uint32_t *)Wpacked, codes, n_segs);
        else if (p.bits == 3) k_unpack_codes<3><<<grid, block, 0, st>>>((const uint32_t *)Wpacked, codes, n_segs);
        else k_unpack_codes<4><<<grid, block, 0, st>>>((const uint32_t *)Wpacked, codes, n_segs);
    }
    if (zcodes != nullptr) {
        const size_t n = (size_t)p.O * p.G;
        const dim3 grid(blocks_for(n)), block(256);
        if (p.bits == 2) k_unpack_z<2><<<grid, block, 0, st>>>((const uint32_t *)zpacked, zcodes, (uint32_t)p.O, (uint32_t)p.G, row_words);
        else if (p.bits == 3) k_unpack_z<3><<<grid, block, 0, st>>>((const uint32_t *)zpacked, zcodes, (uint32_t)p.O, (uint32_t)p.G, row_words);
        else k_unpack_z<4><<<grid, block, 0, st>>>((const uint32_t *)zpacked, zcodes, (uint32_t)p.O, (uint32_t)p.G, row_words);
    }
}

void launch_unpack_work(const Problem &p, const void *work, const void *clampbits, const void *sz, int32_t *codes,
                        uint8_t *clamped, float *zbar, hipStream_t st)
{
    const uint32_t n_segs = (uint32_t)((size_t)p.O * p.I / 32), n_groups = (uint32_t)((size_t)p.O * p.G);    // n_groups <= n_segs
    const dim3 grid(blocks_for(n_segs)), block(256);
    const uint32_t *w = (const uint32_t *)work, *c = (const uint32_t *)clampbits;
    const floatx2 *q = (const floatx2 *)sz;
    if (p.bits == 2) k_unpack_work<2><<<grid, block, 0, st>>>(w, c, q, codes, clamped, zbar, n_segs, n_groups);
    else if (p.bits == 3) k_unpack_work<3><<<grid, block, 0, st>>>(w, c, q, codes, clamped, zbar, n_segs, n_groups);
    else k_unpack_work<4><<<grid, block, 0, st>>>(w, c, q, codes, clamped, zbar, n_segs, n_groups);
}

template <typename WT>
static void init_minmax_t(const InitJob *jobs, int n, hipStream_t st)
{
    const float qmax = (float)((1 << jobs[0].p.bits) - 1);
    // one lane per 8 weights and an xor butterfly over the lanes of a group when every matrix has the same group size
    // of 32 .. 512; one wavefront per group otherwise
    int64_t g = jobs[0].p.g;
    for (int i = 1; i < n; ++i) if (jobs[i].p.g != g) g = 0;
    const bool small = g == 32 || g == 64 || g == 128 || g == 256 || g == 512;
    InitBatch b{};
    uint32_t first = 0;
    for (int i = 0; i < n; ++i) {
        const Problem &p = jobs[i].p;
        b.W[i] = jobs[i].W; b.s[i] = jobs[i].s; b.z[i] = jobs[i].z; b.g[i] = (uint32_t)p.g;
        b.n[i] = small ? (uint32_t)((size_t)p.O * p.I / 8) : (uint32_t)((size_t)p.O * p.G);
        b.first[i] = first;
        first += small ? blocks_for(b.n[i], 256 * kQuantUnroll) : blocks_for(b.n[i], 4);
    }
    for (int i = n; i <= kMaxBatch; ++i) b.first[i] = first;
    const dim3 grid(first), block(256);
    switch (small ? (int)g : 0) {
    case 32:  k_init_minmax_small<WT, 4><<<grid, block, 0, st>>>(b, qmax); break;
    case 64:  k_init_minmax_small<WT, 8><<<grid, block, 0, st>>>(b, qmax); break;
    case 128: k_init_minmax_small<WT, 16><<<grid, block, 0, st>>>(b, qmax); break;
    case 256: k_init_minmax_small<WT, 32><<<grid, block, 0, st>>>(b, qmax); break;
    case 512: k_init_minmax_small<WT, 64><<<grid, block, 0, st>>>(b, qmax); break;
    default:  k_init_minmax_wave<WT><<<grid, block, 0, st>>>(b, qmax);
    }
}

void launch_init_minmax_batch(const InitJob *jobs, int n, hipStream_t st)
{
    if (jobs[0].p.w_bf16) init_minmax_t<bf16_t>(jobs, n, st);
    else init_minmax_t<float>(jobs, n, st);
}

void launch_init_minmax(const Problem &p, const void *W, float *s, float *z, hipStream_t st)
{
    const InitJob j{p, W, s, z};
    launch_init_minmax_batch(&j, 1, st);
}

void launch_reduce_partials(const float *part, float *out, const float *s, size_t n_out, uint32_t n_per, bool scale_by_s,
                            hipStream_t st)
{
    k_reduce_partials<<<dim3(blocks_for(n_out)), dim3(256), 0, st>>>(part, out, s, (uint32_t)n_out, n_per, scale_by_s ? 1 : 0);
}

}  // namespace eqat
