// bf16 MFMA GEMMs of the quantized linear layer (gfx950; fwd and dX on v_mfma_f32_32x32x16_bf16, dW on
// v_mfma_f32_16x16x32_bf16).
//
//   fwd :  Y [T,O]  = X [T,I]  * What[O,I]^T        (K = I)
//   dX  :  dX[T,I]  = dY[T,O]  * What[O,I]          (K = O)
//   dW  :  dWhat^T[I,O] = X[T,I]^T * dY[T,O]        (K = T), fused with the Eq.(3)-(5) epilogue
//
// What is never in HBM: the weight operand of fwd / dX is rebuilt per tile, in registers, from N-bit codes
// (working layout, see WorkCodes) and the (s, zbar) pair of each group, and written to LDS as bf16.
//
// Two LDS tile formats feed the MFMA operands:
//   KC  "K contiguous"  [row][BK + 8]      fragment = one ds_read_b128 per lane
//   KM  "K major"       [k][cols + 32]     fragment = two ds_read_b64_tr_b16 (LDS transpose reads)
// The paddings make both read patterns bank-conflict free.
#include "common.h"
#include "kernels.h"
#include "prof.h"

#include <algorithm>

namespace eqat {

constexpr int kPadKC = 8;    // bf16 elements
constexpr int kPadKM = 32;
constexpr uint32_t kStoreStageBytes = 2048;   // per wave: one 32 x 32 bf16 block of the result on its way out

// ---- fragment reads ---------------------------------------------------------------------------------
// KC tile: lane l supplies row (l % 32), k = kk*16 + (l / 32) * 8 .. + 8
template <int LD>
__device__ __forceinline__ bf16x8 frag_kc(const bf16_t *tile, int row0, int kk, int lane)
{
    return *reinterpret_cast<const bf16x8 *>(tile + (row0 + (lane & 31)) * LD + kk * 16 + (lane >> 5) * 8);
}
// KM tile [k][n] (dX: What with K = O as the slow axis), rows padded by kPadKM.  The producer writes one 16-byte chunk
// per lane and instruction; the 8 (or 4) lanes that fill one row sit 64 bytes apart.  A 128-bit LDS store is served 8
// lanes per cycle over 32 four-byte banks (the model that reproduces the SQ_LDS_BANK_CONFLICT readings of every layout
// tried here: 24 extra cycles per store unswizzled, 8 with a swizzle that only separated lanes 4 apart, 0 for the
// forward kernel's [n][k] tile), so lanes 128 bytes apart in one row share their banks.  The four chunks of every
// 32-column block are therefore XOR-permuted with km_chunk_swz(k, block): blocks two apart, and the blocks that a
// second row of the same store cycle puts on the same banks, get different chunk positions.
__device__ __forceinline__ int km_chunk_swz(int k, int colblock) { return ((colblock >> 1) + 2 * (k & 1)) & 3; }

// The transpose read hands lane i (of each 16-lane block) four k-consecutive values of column i, gathered from the lanes
// that addressed rows k..k+3.  Block b = lane/16: columns 16*(b&1).., k half b>>1.
template <int LD>
__device__ __forceinline__ bf16x8 frag_km(const bf16_t *tile, int col0, int kk, int lane)
{
    const int i = lane & 15, b = lane >> 4;
    const int k = kk * 16 + (b >> 1) * 8 + (i >> 2), col = col0 + (b & 1) * 16 + (i & 3) * 4;
    const int pcol = (col & ~31) | ((((col >> 3) & 3) ^ km_chunk_swz(k, col >> 5)) << 3) | (col & 7);
    const bf16_t *p = tile + k * LD + pcol;
    typedef short4v __attribute__((address_space(3))) * lds_p;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p + 4 * LD));      // (k + 4) & 3 == k & 3: same permutation
    typedef short short8v __attribute__((ext_vector_type(8)));
    short8v r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// ---- workgroup -> tile mapping ---------------------------------------------------------------------------
// Consecutive workgroup ids go round-robin over the 8 XCDs, each with its own L2.  Give every XCD a
// contiguous range of tile ids, then walk the tiles in bands of kBand tile-rows so that the tiles resident on
// one XCD at a time share their operand panels.
// nb = number of tiles; (xcd, loc) = the loc-th tile of XCD xcd.  Returns false past the end of that XCD's range.
__host__ __device__ __forceinline__ bool tile_of_xcd_slot(int nb, int xcd, int loc, int tiles_m, int tiles_n, int &tm, int &tn, int kBand)
{
    const int per = nb >> 3, rem = nb & 7;
    if (loc >= per + (xcd < rem ? 1 : 0)) return false;
    const int pid = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + loc;
    const int width = kBand * tiles_n, band = pid / width, first = band * kBand;
    const int rows = tiles_m - first < kBand ? tiles_m - first : kBand, in = pid - band * width;
    tm = first + in % rows;
    tn = in / rows;
    return true;
}
// one tile per workgroup
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int &tm, int &tn, int kBand = 8)
{
    (void)tile_of_xcd_slot((int)gridDim.x, (int)(blockIdx.x & 7), (int)(blockIdx.x >> 3), tiles_m, tiles_n, tm, tn, kBand);
}

// ---- work of one workgroup: whole tiles, then a share of the tiles that do not fill a round ---------------
// A grid of G workgroups (all resident at once, G / 8 per XCD) covers nb tiles.  When nb is between one and two rounds
// of G (the 13B-shaped linears at 4096 tokens give 1.25 rounds of 256 x 256 tiles) the second round would run on a
// fraction of the chip.  Instead the tiles beyond the last whole round but one are cut along K: their K-tile pairs,
// laid end to end per XCD, are dealt out in equal contiguous runs, so a workgroup's run may begin and end in the middle
// of a tile.  A run is at least one tile long, so a tile has at most two contributors.  The contributor that arrives
// first writes its fp32 accumulators to memory and raises the tile's flag; the one that arrives second waits for the
// flag (a wait for a workgroup that is already running and itself waits for nobody), adds that part to its own
// accumulators (a + b = b + a: the result does not depend on who came first) and runs the tile's epilogue.  Counter
// and flag of a tile are back at zero when its second contributor is done, so a launch leaves them as it found them.
// Whether cutting pays is a measured matter (host side, plan_tiles): a partly filled round costs less than its share
// of a full one on this power-limited chip, and every part costs a trip of 256 KB through memory.
// When the tiles beyond the first round are few (at most half a round), dealing out runs would cut nearly every tile of
// the launch (1.25 rounds: 31 of 40 per XCD).  Then (`split`) every workgroup first computes one whole tile, and each
// of the remaining tiles is shared by c = W / n_sk workgroups (at most kSkMaxSplit), a c-th of its K range each; all
// write their parts and the one that arrives last adds them up in their order (a fixed order: reproducible).
constexpr int kSkMaxSplit = 8;
struct SkPlan {
    int walk;              // 0: the grid has one workgroup per tile and none of the below applies
    int dp_rounds;         // whole tiles per workgroup: tiles loc0 + r * (G / 8) of its XCD, r < dp_rounds
    int split;             // 1: the tiles beyond the whole rounds are split among groups of workgroups (see above)
    int pairs;             // K-tile pairs per output tile
    float *partials;       // [G][2] accumulator tiles (a run has at most a head and a tail piece)
    uint32_t *counters;    // [2][2 G], zero: arrivals, then flags, one each per tile that may be cut (at most 2 G / 8 per XCD)
};
struct SkItem {
    int tm, tn, ctr;       // tile, and the index of its counter when it is cut
    int kb, ke;            // K-tile pairs [kb, ke) of the tile
    int parts, first;      // number of contributors (1: the whole tile is mine) and the first one's index in the XCD
    int first_slot;        // which of its two buffers the first contributor used (all others use buffer 0)
    int fixed;             // 1: a split tile (all contributors write, the last one to arrive sums all parts); 0: a run's tile
};
__host__ __device__ __forceinline__ int sk_owner_of_pair(int p, int base, int extra)
{
    const int cut = extra * (base + 1);
    return p < cut ? p / (base + 1) : extra + (p - cut) / (base > 0 ? base : 1);
}
// item number j of workgroup `bid` of a grid of `grid`; false past its last one
__host__ __device__ __forceinline__ bool sk_item_of(const SkPlan &sk, int nb, int tiles_m, int tiles_n, int band, int bid, int grid,
                                                   int j, SkItem &it)
{
    const int xcd = bid & 7, loc0 = bid >> 3;
    it.kb = 0; it.ke = sk.pairs; it.parts = 1; it.first = 0; it.first_slot = 0; it.ctr = 0; it.fixed = 0;
    if (!sk.walk) return j == 0 && tile_of_xcd_slot(grid, xcd, loc0, tiles_m, tiles_n, it.tm, it.tn, band);
    const int W = grid >> 3;
    if (j < sk.dp_rounds) return tile_of_xcd_slot(nb, xcd, loc0 + j * W, tiles_m, tiles_n, it.tm, it.tn, band);
    const int n_sk = (nb >> 3) + (xcd < (nb & 7) ? 1 : 0) - sk.dp_rounds * W;
    if (n_sk <= 0) return false;
    if (sk.split) {
        if (j != sk.dp_rounds) return false;                       // one piece per workgroup
        const int c = W / n_sk < kSkMaxSplit ? W / n_sk : kSkMaxSplit;                   // contributors per tile (at least 2: the host's choice)
        const int t = loc0 / c, me = loc0 - t * c;
        if (t >= n_sk) return false;
        const int base = sk.pairs / c, extra = sk.pairs % c;
        it.kb = me * base + (me < extra ? me : extra);
        it.ke = it.kb + base + (me < extra ? 1 : 0);
        it.parts = c; it.first = t * c; it.fixed = 1;
        it.ctr = xcd * 2 * W + t;
        return tile_of_xcd_slot(nb, xcd, sk.dp_rounds * W + t, tiles_m, tiles_n, it.tm, it.tn, band);
    }
    const int P = sk.pairs, total = n_sk * P, base = total / W, extra = total % W;
    const int start = loc0 * base + (loc0 < extra ? loc0 : extra), end = start + base + (loc0 < extra ? 1 : 0);
    const int t = start / P + (j - sk.dp_rounds);
    if (start >= end || t * P >= end) return false;
    it.kb = (start > t * P ? start : t * P) - t * P;
    it.ke = (end < (t + 1) * P ? end : (t + 1) * P) - t * P;
    if (it.kb > 0 || it.ke < P) {
        it.first = sk_owner_of_pair(t * P, base, extra);
        it.parts = sk_owner_of_pair((t + 1) * P - 1, base, extra) - it.first + 1;
        const int fstart = it.first * base + (it.first < extra ? it.first : extra);
        it.first_slot = fstart / P == t ? 0 : 1;
        it.ctr = xcd * 2 * W + t;          // t < n_sk <= 2 W: the plan never cuts more than two rounds
    }
    return tile_of_xcd_slot(nb, xcd, sk.dp_rounds * W + t, tiles_m, tiles_n, it.tm, it.tn, band);
}
__device__ __forceinline__ bool sk_item(const SkPlan &sk, int nb, int tiles_m, int tiles_n, int band, int j, SkItem &it)
{
    return sk_item_of(sk, nb, tiles_m, tiles_n, band, (int)blockIdx.x, (int)gridDim.x, j, it);
}

// A contributor of a tile cut along K is done with its K range.  Returns true in the one that holds the sum of all
// parts in `acc` afterwards and runs the tile's epilogue, false in the others (their part is in memory, their work on
// the tile done).
//   Two contributors of a run: the one that arrives first writes its part and raises the tile's flag, the one that
//   arrives second waits for the flag (for a workgroup that is already running and itself waits for nobody) and adds
//   that part to its own accumulators (a + b = b + a).
//   A split tile (it.fixed): every contributor writes its part and counts itself in; the one that finds itself last
//   adds up ALL parts from memory, its own included, in the order of the contributors.  Nobody waits for anybody, and
//   the sum does not depend on who came last.
// Layout of a part: the float4 number q of accumulator block (i, j) of thread t at ((i * NI + j) * 4 + q) * NT + t.
// The contributors may sit on different XCDs, each with its own L2, so parts and flag are written and read with
// device-scope accesses (cache policy sc1: written through to memory, read from memory); no cache is flushed or
// invalidated as a whole (a device-scope fence writes back and invalidates the entire L2 of the XCD, operand panels
// included: measured, that alone cost more than cutting the tiles gained).  Order on the writing side: every wave
// waits for its stores to complete, the workgroup meets, then one thread signals.
constexpr int kAuxDeviceScope = 16;      // "sc1" of the raw buffer intrinsics on gfx940 and later
constexpr int kSkSpinLimit = 1 << 22;    // polls of ~1 us: a bound that is never reached, so that no wave can spin for ever
__device__ __forceinline__ void wait_all_and_barrier();
// register r of block (i, j), whichever way a kernel keeps its accumulators
template <int MI, int NI> __device__ __forceinline__ float acc_get(const floatx16 (&acc)[MI][NI], int i, int j, int r) { return acc[i][j][r]; }
template <int MI, int NI> __device__ __forceinline__ float acc_get(const floatx4 (&acc)[MI][NI][4], int i, int j, int r) { return acc[i][j][r >> 2][r & 3]; }
template <int MI, int NI> __device__ __forceinline__ void acc_set(floatx16 (&acc)[MI][NI], int i, int j, int r, float v) { acc[i][j][r] = v; }
template <int MI, int NI> __device__ __forceinline__ void acc_set(floatx4 (&acc)[MI][NI][4], int i, int j, int r, float v) { acc[i][j][r >> 2][r & 3] = v; }
// NB = 32 x 32 blocks of a part that are fetched together (16 registers each)
template <int MI, int NI, int NT, int NB = 2, typename ACC>
__device__ __forceinline__ bool sk_hand_in(const SkPlan &sk, const SkItem &it, ACC &acc, int tid)
{
    static_assert((MI * NI) % NB == 0, "whole batches");
    __shared__ uint32_t s_sums;
    constexpr size_t kTile = (size_t)MI * NI * 16 * NT;          // floats per part
    constexpr uint32_t kTileBytes = (uint32_t)(kTile * sizeof(float));
    const int xcd = (int)(blockIdx.x & 7), me = (int)(blockIdx.x >> 3) - it.first;       // 0 .. parts - 1
    const bool split = it.fixed != 0;
    uint32_t *arrivals = sk.counters + it.ctr, *flag = sk.counters + 2 * (int)gridDim.x + it.ctr;
    if (tid == 0) s_sums = split ? 0u : atomicInc(arrivals, 1u);                          // run: 0 -> 1 -> 0
    __syncthreads();
    const bool second = s_sums != 0u;              // of a run
    // Straight-line code for all roles (branches around the accumulators make the register allocator spill them): the
    // stores of the contributor that keeps its part in registers go to an out-of-range offset, where they are dropped.
    const uint32_t st_base = second ? kOobOffset : (uint32_t)tid * 16u;
    const __amdgpu_buffer_rsrc_t mine =
        make_rsrc(sk.partials + ((size_t)blockIdx.x * 2 + (!split && me == 0 ? it.first_slot : 0)) * kTile, kTileBytes);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                intx4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = __float_as_int(acc_get<MI, NI>(acc, i, j, 4 * q + e));
                __builtin_amdgcn_raw_buffer_store_b128(v, mine, st_base + (uint32_t)(((i * NI + j) * 4 + q) * NT * 16), 0, kAuxDeviceScope);
            }
            __builtin_amdgcn_sched_barrier(0);      // one 32 x 32 block at a time: few register copies
        }
    wait_all_and_barrier();                // every store of the workgroup has completed
    if (tid == 0) {
        if (split) {
            const uint32_t before = __hip_atomic_fetch_add(arrivals, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const bool last = before == (uint32_t)(it.parts - 1);
            if (last) __hip_atomic_store(arrivals, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_sums = last ? 1u : 0u;
        } else if (!second) {
            __hip_atomic_store(flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            int polls = 0;
            while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u && ++polls < kSkSpinLimit)
                __builtin_amdgcn_s_sleep(32);
            __hip_atomic_store(flag, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
    const bool sums = s_sums != 0u;
    // the last contributor of a split tile starts from zero and takes every part, its own too, from memory (bitwise AND
    // instead of a branch, see above)
    const uint32_t keep = (split && sums) ? 0u : ~0u;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_set<MI, NI>(acc, i, j, r, __uint_as_float(__float_as_uint(acc_get<MI, NI>(acc, i, j, r)) & keep));
    // parts to add, in the order of the contributors (a trip count of zero for those that do not sum)
    const int n_take = !sums ? 0 : split ? it.parts : 1;
    for (int k = 0; k < n_take; ++k) {
        const int from = split ? it.first + k : it.first + (1 - me);                  // contributor whose part this is
        const int slot = (!split && me == 1) ? it.first_slot : 0;
        const __amdgpu_buffer_rsrc_t theirs = make_rsrc(sk.partials + (((size_t)from * 8 + xcd) * 2 + slot) * kTile, kTileBytes);
        // NB blocks in flight at a time.  In the fwd / dX kernels two (32 registers): with more (two parts together, 64
        // registers) they spilled or lost their second workgroup per CU, because the pipeline state of the next tile is
        // alive here.
#pragma unroll
        for (int b0 = 0; b0 < MI * NI; b0 += NB) {
            intx4 v[NB][4];
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    v[b][q] = __builtin_amdgcn_raw_buffer_load_b128(theirs, (uint32_t)tid * 16u + (uint32_t)(((b0 + b) * 4 + q) * NT * 16), 0, kAuxDeviceScope);
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        acc_set<MI, NI>(acc, (b0 + b) / NI, (b0 + b) % NI, 4 * q + e,
                                        acc_get<MI, NI>(acc, (b0 + b) / NI, (b0 + b) % NI, 4 * q + e) + __int_as_float(v[b][q][e]));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    return sums;
}

// ======================================================================================================
// fwd / dX:  C[M,N] = A[M,K] * B,  A plain bf16 (K contiguous), B = What rebuilt from codes.
//   BT = false (fwd): B element (k, n) = What[n][k]   -> weight tile is KC  [BN][BK]
//   BT = true  (dX) : B element (k, n) = What[k][n]   -> weight tile is KM  [BK][BN]
// ======================================================================================================
struct GemmQArgs {
    const bf16_t *A; const uint32_t *codes; const floatx2 *sz; bf16_t *C;
    int M, N, K;           // problem
    int I, G, g;           // weight matrix geometry: row length, groups per row, group size
    uint32_t a_bytes, codes_bytes, sz_bytes, c_bytes;
    int tiles_m, tiles_n;
    int band;              // tile rows walked together by one XCD (see tile_of_xcd_slot)
    SkPlan sk;             // which tiles, or parts of tiles, a workgroup computes
};

template <int V> struct IC { static constexpr int value = V; };
// f(IC<0>{}), f(IC<1>{}), ..., f(IC<N - 1>{}): a loop whose index is a compile-time constant inside the body
template <int N, int I = 0, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) { f(IC<I>{}); static_for<N, I + 1>(f); }
}

// With more than 128 accumulator registers per lane the accumulators must live in AGPRs (the MFMA "acd" form);
// the compiler only picks that form when it believes the kernel needs AGPRs, which this empty statement asserts.
template <int ACC_REGS> __device__ __forceinline__ void want_agpr_accumulators()
{
    if constexpr (ACC_REGS > 128) { float zero = 0.0f; asm volatile("" ::"a"(zero)); }
}

// ---- KC tile filled by buffer loads that write LDS directly ----------------------------------------------
// Such a load puts the 16 bytes of lane j at (wave-uniform LDS base) + 16*j, so one instruction fills 8 rows of
// a [rows][64] bf16 tile and no padding can be placed inside it.  Bank conflicts of the fragment reads are
// avoided by a swizzle instead: the 16-byte chunk c of row r lives at position c ^ ((r >> 1) & 7); the
// permutation is applied on the global-address side, which is free.
__device__ __forceinline__ int kc_swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

__device__ __forceinline__ bf16x8 frag_kc_swz(const bf16_t *tile, int row0, int kk, int lane)
{
    const int r = row0 + (lane & 31);
    return *reinterpret_cast<const bf16x8 *>(tile + r * 64 + kc_swz(r, kk * 2 + (lane >> 5)) * 8);
}

// 16 bytes per lane from a buffer straight into LDS: lane j's bytes land at lds_wave_base + 16 j; a voffset beyond the
// buffer writes zeros.  Issued as inline assembly on purpose: the compiler models the builtin form as a store to LDS and,
// not being able to tell it apart from the transpose reads of the other buffer, waits for vmcnt(0) before the next LDS
// read, which puts the whole fetch latency on the critical path of every K tile.  Nothing tracks these loads, so every
// consumer sits behind an explicit "s_waitcnt vmcnt(0)" + barrier (the one in the main loop, and the one after it).
struct RawRsrc { intx4 w; };
__device__ __forceinline__ RawRsrc make_raw_rsrc(const void *p, uint32_t bytes)
{
    const uint64_t a = (uint64_t)p;
    RawRsrc r;
    r.w[0] = (int)(uint32_t)a; r.w[1] = (int)(uint32_t)((a >> 32) & 0xFFFFu); r.w[2] = (int)bytes; r.w[3] = 0x00020000;
    return r;
}
// The LDS destination is a 32-bit LDS address that the caller has built from wave-uniform scalars (so that M0 costs
// one scalar instruction instead of a 64-bit pointer computation and a v_readfirstlane per load).
__device__ __forceinline__ uint32_t lds_addr_of(const void *p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)p;
}
__device__ __forceinline__ void load_to_lds16_at(const RawRsrc &r, uint32_t lds_addr_uniform, uint32_t voffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_addr_uniform), "v"(voffset), "s"(r.w) : "memory", "m0");
}

// Workgroup barrier behind "everything I issued has completed".  The wait is the builtin, not assembly text, so that the
// compiler's own wait-count bookkeeping knows that its register loads are complete here and inserts no further vmcnt
// wait while the (untracked) direct-to-LDS loads of the next tile are in flight: such a wait counts ALL outstanding
// loads and would stall on the tile fetch.  The empty asm statements keep the compiler from moving LDS accesses across.
__device__ __forceinline__ void wait_all_and_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0070);       // vmcnt(0) lgkmcnt(0); expcnt field at its maximum = no wait
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Software pipeline of the main loop (one workgroup, K tile kt, LDS buffer kt & 1):
//   - behind the barrier of tile kt (which sits before its last 16-wide slice) the activation tile kt+2 starts to
//     stream from global memory straight into LDS buffer kt & 1, whose last fragments are in registers by then;
//   - the weight codes and (s, zbar) pairs of tile kt+3 are fetched into registers (two staging sets);
//   - while the MFMAs consume buffer kt & 1, the staged codes of tile kt+1 become bf16 What in the other weight
//     buffer, a quarter after each slice, so that this VALU / LDS-write work hides under the MFMAs of the same
//     wave; fragments of slice kk+1 are read while slice kk multiplies.
// K tiles past the end of K multiply zeros: the weights there are exactly zero (see load_a below).
// A workgroup may own several output tiles; the pipeline then runs on through the tile boundaries.
// CUT: the instantiation for launches that cut tiles along K (SkPlan::dp_rounds == 0, or split, with walk) or whose contraction
// length is not a multiple of two K tiles; the other one carries none of that code (the main loop is sensitive to it).
template <int BITS, bool BT, bool CUT, int BM, int BN, int BK, int WGM, int WGN>
__global__ __launch_bounds__(64 * WGM * WGN) void k_gemm_q(const GemmQArgs a)
{
    constexpr int NT = 64 * WGM * WGN, NW = WGM * WGN, WTM = BM / WGM, WTN = BN / WGN, MI = WTM / 32, NI = WTN / 32;
    constexpr int LDB = BT ? BN + kPadKM : BK + kPadKC;
    constexpr uint32_t kRingBytes = 2u * (uint32_t)(BM * BK + (BT ? BK * LDB : BN * LDB)) * 2u;    // the two K-tile buffers
    constexpr int A_ELEMS = BM * BK, B_ELEMS = BT ? BK * LDB : BN * LDB;
    constexpr int A_LOADS = BM / 8 / NW;              // direct-to-LDS instructions per wave (8 rows each)
    constexpr int B_SEGS = BN * BK / 32 / NT;         // 32-code segments per thread
    constexpr int KK = BK / 16;
    static_assert(BK == 64 && BM % (8 * NW) == 0 && BN * BK / 32 % NT == 0, "tile / thread mismatch");

    want_agpr_accumulators<MI * NI * 16>();
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t *sA = reinterpret_cast<bf16_t *>(smem_raw);            // [2][A_ELEMS]
    bf16_t *sB = sA + 2 * A_ELEMS;                                // [2][B_ELEMS]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    // Items of this workgroup (see SkPlan): whole tiles, then possibly pieces of tiles cut along K.  The K loop runs
    // THROUGH the item boundaries: the loaders below each keep their own position in that sequence, two (activations)
    // and three (codes) K tiles ahead of the MFMAs, so that the first K tiles of the next item are in LDS and in
    // registers when the last MFMA of the current one issues.
    const int ntiles = a.tiles_m * a.tiles_n;
    const int nk = (a.K + BK - 1) / BK, nk2 = (nk + 1) & ~1;              // K tiles per output tile, two per trip
    // item j: origin of its tile, first K tile and number of K tiles (even); past the last item: rows and columns out
    // of range (the loaders then fetch zeros)
    const int grid = (int)gridDim.x, xcd = (int)(blockIdx.x & 7), loc0 = (int)(blockIdx.x >> 3);
    const int loc_step = a.sk.walk ? grid >> 3 : ntiles;          // no second tile without a.sk.walk
    auto item_of = [&](int j, SkItem &it, int &m0, int &n0) -> bool {
        bool ok;
        if constexpr (CUT) {
            ok = sk_item(a.sk, ntiles, a.tiles_m, a.tiles_n, a.band, j, it);
            if (!ok) { it.kb = 0; it.ke = nk2 / 2; it.parts = 1; }
        } else {
            // whole tiles only: tile loc0 + j * (G / 8) of this XCD's range (walk), or the one tile of this workgroup
            ok = tile_of_xcd_slot(a.sk.walk ? ntiles : grid, xcd, loc0 + j * loc_step, a.tiles_m, a.tiles_n, it.tm, it.tn, a.band);
            it.kb = 0; it.ke = nk2 / 2; it.parts = 1;
        }
        m0 = ok ? it.tm * BM : a.tiles_m * BM;
        n0 = ok ? it.tn * BN : a.tiles_n * BN;
        return ok;
    };

    const RawRsrc rA = make_raw_rsrc(a.A, a.a_bytes);
    const __amdgpu_buffer_rsrc_t rCst = make_rsrc(a.C, a.c_bytes);
    const __amdgpu_buffer_rsrc_t rC = make_rsrc(a.codes, a.codes_bytes);
    const __amdgpu_buffer_rsrc_t rS = make_rsrc(a.sz, a.sz_bytes);
    const uint32_t code_row_bytes = (uint32_t)a.I / 32u * (4u * WorkCodes<BITS>::kWords);

    WorkCodes<BITS> stC[2][B_SEGS];
    floatx2 stS[2][B_SEGS];
    WhatTable<BITS> tabs[2][B_SEGS];

    // Activation tiles stream into LDS strictly in order (k0 = 0, BK, 2 BK, ... of one output tile, then of the next):
    // every direct-to-LDS instruction keeps a running byte offset that advances by one tile row segment per call, and
    // M0 comes from wave-uniform scalars.  Columns past K of a row would read the start of the next row; they meet weights
    // that are exactly zero (step size and zero point of a column past the end load as 0), and are not loaded at all when
    // K is ragged (see k_ragged below).
    const uint32_t ldsA = lds_addr_of(sA);
    uint32_t offA[A_LOADS];
    int a_tile = 0, a_left = 0;                     // loader position: tile ordinal, K tiles left in it
    // When K is not a multiple of two K tiles, the last K tile of an output tile reaches past the end of its rows (and a
    // padding K tile lies past it altogether).  The weights there are zero, but 0 * Inf is NaN: a non-finite value in
    // row t + 1 must not leak into row t, so the chunks past K of those tiles are loaded from out of range (zeros).
    const bool k_ragged = CUT && a.K % (2 * BK) != 0;      // wave-uniform; the host sends every such K to this instantiation
    int a_kt = 0;                                   // K tile (within its output tile) that the next load_a fetches
    uint32_t a_past_k = 0;                          // bit `it`: in K tile nk - 1, this lane's chunk of load `it` lies past K
    if (k_ragged) {
        const int tail_cols = a.K - (nk - 1) * BK;  // 8 .. 64 valid columns in K tile nk - 1
#pragma unroll
        for (int it = 0; it < A_LOADS; ++it) {
            const int row = (wave * A_LOADS + it) * 8 + (lane >> 3);
            if (kc_swz(row, lane & 7) * 8 >= tail_cols) a_past_k |= 1u << it;
        }
    }
    auto a_enter_tile = [&]() {
        int m0, n0;
        SkItem si;
        (void)item_of(a_tile, si, m0, n0);
#pragma unroll
        for (int it = 0; it < A_LOADS; ++it) {
            const int row = (wave * A_LOADS + it) * 8 + (lane >> 3);
            const uint64_t o = ((uint64_t)(m0 + row) * (uint64_t)a.K + (uint64_t)((CUT ? si.kb * 2 * BK : 0) + kc_swz(row, lane & 7) * 8)) * 2u;
            offA[it] = o < kOobOffset ? (uint32_t)o : kOobOffset;   // rows past the matrix stay out of range for good
        }
        a_left = CUT ? 2 * (si.ke - si.kb) : nk2;
        a_kt = CUT ? 2 * si.kb : 0;
        ++a_tile;
    };
    auto load_a = [&](int buf) {
        --a_left;
        if (k_ragged && a_kt >= nk - 1) {            // rare: the last (and the padding) K tile of a ragged K
            const uint32_t past = a_kt >= nk ? ~0u : a_past_k;
#pragma unroll
            for (int it = 0; it < A_LOADS; ++it) {
                load_to_lds16_at(rA, ldsA + (uint32_t)((buf * A_ELEMS + (wave * A_LOADS + it) * 8 * 64) * 2),
                                 (past >> it) & 1u ? kOobOffset : offA[it]);
                offA[it] += BK * 2;
            }
        } else {
#pragma unroll
            for (int it = 0; it < A_LOADS; ++it) {
                load_to_lds16_at(rA, ldsA + (uint32_t)((buf * A_ELEMS + (wave * A_LOADS + it) * 8 * 64) * 2), offA[it]);
                offA[it] += BK * 2;
            }
        }
        ++a_kt;
    };
    // Weight codes and (s, zbar) pairs, in the same order.  Forward: a segment's group index wcol / g is carried from
    // call to call (a K tile advances wcol by BK <= 2 g, so two conditional steps replace a division per K tile).
    int grp[B_SEGS], rem[B_SEGS];
    int c_tile = 0, c_left = 0, c_n0 = 0, c_k0 = 0;
    auto c_enter_tile = [&]() {
        int m0;
        SkItem si;
        (void)item_of(c_tile, si, m0, c_n0);
        c_k0 = CUT ? si.kb * 2 * BK : 0;
#pragma unroll
        for (int it = 0; it < B_SEGS; ++it) {
            const int sidx = it * NT + tid;
            const int wcol = BT ? c_n0 + (sidx % (BN / 32)) * 32 : c_k0 + (sidx % (BK / 32)) * 32;
            grp[it] = wcol / (int)a.g;
            rem[it] = wcol % (int)a.g;
        }
        c_left = CUT ? 2 * (si.ke - si.kb) : nk2;
        ++c_tile;
    };
    auto load_codes = [&](auto set) {
        constexpr int S = decltype(set)::value;
        --c_left;
#pragma unroll
        for (int it = 0; it < B_SEGS; ++it) {
            const int sidx = it * NT + tid;
            int wrow, wcol;   // position in the weight matrix [O][I]
            if (!BT) { wrow = c_n0 + sidx / (BK / 32); wcol = c_k0 + (sidx % (BK / 32)) * 32; }
            else     { wrow = c_k0 + sidx / (BN / 32); wcol = c_n0 + (sidx % (BN / 32)) * 32; }
            const bool ok = wcol < a.I;
            stC[S][it] = load_work_codes<BITS>(rC, (uint32_t)wrow * code_row_bytes + (uint32_t)(wcol >> 5) * (4u * WorkCodes<BITS>::kWords));
            const intx2 sv = buf_load8(rS, ok ? ((uint32_t)wrow * (uint32_t)a.G + (uint32_t)grp[it]) * 8u : kOobOffset);
            stS[S][it][0] = __int_as_float(sv[0]);
            stS[S][it][1] = __int_as_float(sv[1]);
            if (!BT) {
#pragma unroll
                for (int h = 0; h < BK / 32; ++h) {
                    rem[it] += 32;
                    const bool wrap = rem[it] >= (int)a.g;
                    rem[it] = wrap ? rem[it] - (int)a.g : rem[it];
                    grp[it] += wrap ? 1 : 0;
                }
            }
        }
        c_k0 += BK;
    };
    // A loader steps into the next output tile BETWEEN K steps (and between the loads of the start-up sequence): a
    // branch inside a K step would cut the instruction schedule of the step in two.
    auto loaders_advance = [&]() {
        if (a_left == 0) a_enter_tile();
        if (c_left == 0) c_enter_tile();
    };
    // piece P of KK: every KK-th 16-byte store of the staged weight tile
    auto commit_piece = [&](auto set, auto piece, int buf) {
        constexpr int S = decltype(set)::value, P = decltype(piece)::value;
        bf16_t *dB = sB + buf * B_ELEMS;
#pragma unroll
        for (int it = 0; it < B_SEGS; ++it) {
            const int sidx = it * NT + tid;
            int r, c;
            if (!BT) { r = sidx / (BK / 32); c = (sidx % (BK / 32)) * 32; }
            else     { r = sidx / (BN / 32); c = (sidx % (BN / 32)) * 32; }
            WhatTable<BITS> &tab = tabs[S][it];
            if constexpr (P == 0) tab.build(stS[S][it][0], stS[S][it][1]);     // piece 0 of a tile always runs first
            bf16x8 *dst = reinterpret_cast<bf16x8 *>(dB + r * LDB + c);
            const int sw = BT ? km_chunk_swz(r, c >> 5) : 0;                    // KM tile: see km_chunk_swz
            if ((it * 4 + 0) % KK == P) dst[0 ^ sw] = tab.template eight<0>(stC[S][it]);
            if ((it * 4 + 1) % KK == P) dst[1 ^ sw] = tab.template eight<1>(stC[S][it]);
            if ((it * 4 + 2) % KK == P) dst[2 ^ sw] = tab.template eight<2>(stC[S][it]);
            if ((it * 4 + 3) % KK == P) dst[3 ^ sw] = tab.template eight<3>(stC[S][it]);
        }
    };

    floatx16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    bf16x8 fa[2][MI], fb[2][NI];
    // B fragments first: the MFMAs run i-major, so both B fragments and A0 are needed by the first two MFMAs of a
    // slice and A3 only by the seventh; issued in that order, one read per MFMA of the previous slice, every read gets
    // about a slice of latency budget.
    auto read_frags = [&](int slot, const bf16_t *cA, const bf16_t *cB, int kk) {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            if (!BT) fb[slot][j] = frag_kc<LDB>(cB, wn * WTN + j * 32, kk, lane);
            else     fb[slot][j] = frag_km<LDB>(cB, wn * WTN + j * 32, kk, lane);
        }
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[slot][i] = frag_kc_swz(cA, wm * WTM + i * 32, kk, lane);
    };
    // One K tile.  PAR = kt & 1 is the LDS buffer being multiplied.  On entry the fragments of slice 0 are already
    // in registers.  The barrier sits BEFORE the MFMAs of the last slice: by then every wave has issued all its LDS
    // reads of this tile and finished writing the next one, so after the barrier the next tile's first fragments and
    // the global loads for later tiles are started and their latency hides under the last slice's MFMAs.
    auto mfma_slice = [&](int slot) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
    };
    auto step = [&](auto par) {
        constexpr int PAR = decltype(par)::value;
        const bf16_t *cA = sA + PAR * A_ELEMS, *cB = sB + PAR * B_ELEMS;
        // stage kk: start the reads of slice kk+1, multiply slice kk, convert a quarter of the next weight tile
        auto interleave = [&]() {
            // pipeline hint for the scheduler: one MFMA, one fragment read of the next slice, a few VALU ops of the
            // conversion, repeated (LDS reads spread over the slice measure 2-5 % faster than a burst in front of it)
#pragma unroll
            for (int q = 0; q < MI * NI; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);
            }
        };
        read_frags(1, cA, cB, 1);
        mfma_slice(0);
        commit_piece(IC<PAR ^ 1>{}, IC<1>{}, PAR ^ 1);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(0, cA, cB, 2);
        mfma_slice(1);
        commit_piece(IC<PAR ^ 1>{}, IC<2>{}, PAR ^ 1);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(1, cA, cB, 3);
        mfma_slice(0);
        commit_piece(IC<PAR ^ 1>{}, IC<3>{}, PAR ^ 1);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        wait_all_and_barrier();   // next activation tile landed, my LDS traffic done
        // last slice of this tile, overlapped with the start of the next two tiles.  (The codes fetched here are first
        // used behind the next barrier, so the compiler never needs a vmcnt wait while the activation loads fly.)
        load_a(PAR);
        read_frags(0, sA + (PAR ^ 1) * A_ELEMS, sB + (PAR ^ 1) * B_ELEMS, 0);
        mfma_slice(1);
        commit_piece(IC<PAR>{}, IC<0>{}, PAR);
        interleave();
        load_codes(IC<PAR ^ 1>{});
        __builtin_amdgcn_sched_barrier(0);
    };

    // start-up of the first tile: K tiles 0 and 1 of the activations, 0, 1 and 2 of the codes, weight tile 0 rebuilt
    loaders_advance();
    load_codes(IC<0>{});
    load_a(0);
    loaders_advance();
    load_codes(IC<1>{});
    commit_piece(IC<0>{}, IC<0>{}, 0);
    commit_piece(IC<0>{}, IC<1>{}, 0);
    commit_piece(IC<0>{}, IC<2>{}, 0);
    commit_piece(IC<0>{}, IC<3>{}, 0);
    wait_all_and_barrier();
    loaders_advance();
    load_codes(IC<0>{});
    load_a(1);
    commit_piece(IC<1>{}, IC<0>{}, 1);
    read_frags(0, sA, sB, 0);

    for (int jt = 0;; ++jt) {
        int m0, n0;
        SkItem si;
        if (!item_of(jt, si, m0, n0)) break;
        // Two K tiles per trip, unconditionally (the register staging sets alternate at compile time, and a branch
        // between the two halves makes the accumulators flow through a merge that costs hundreds of copies).  With an
        // odd K-tile count the extra tile lies past K and multiplies zeros.  The last trips of this loop already fetch
        // (and rebuild) the first K tiles of the next item.
        for (int kt = CUT ? 2 * si.kb : 0; kt < (CUT ? 2 * si.ke : nk2); kt += 2) {
            loaders_advance();
            step(IC<0>{});
            loaders_advance();
            step(IC<1>{});
        }
        // a tile cut along K: only the contributor that arrives last stores it, from the sum of all parts
        bool mine_to_store = true;
        if constexpr (CUT) mine_to_store = si.parts == 1 || sk_hand_in<MI, NI, NT>(a.sk, si, acc, tid);
        if (!mine_to_store) {
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
            continue;
        }

        // C[m][n]: lane holds column n = l % 32 and rows 8*(r/4) + 4*(l/32) + r%4 of each 32x32 block.  Stored from
        // the registers that is sixteen 2-byte stores per block, each to two rows; instead the block goes through a
        // 2 KB patch of LDS of the wave's own (behind the tile ring, which the loads of the next tile are filling) and
        // leaves as two 16-byte stores per lane, 64 bytes of a row from four neighbouring lanes.
        {
            unsigned char *const stg = smem_raw + kRingBytes + wave * kStoreStageBytes;
            bf16_t *const cell = reinterpret_cast<bf16_t *>(stg) + (lane >> 5) * (4 * 32) + (lane & 31);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        cell[(8 * (r >> 2) + (r & 3)) * 32] = (bf16_t)acc[i][j][r];
                        acc[i][j][r] = 0.0f;
                    }
                    asm volatile("" ::: "memory");
                    __builtin_amdgcn_wave_barrier();       // LDS accesses of a wave complete in order
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        const intx4 v = *reinterpret_cast<const intx4 *>(stg + k * 1024 + lane * 16);
                        const int m = m0 + wm * WTM + i * 32 + k * 16 + (lane >> 2), n = n0 + wn * WTN + j * 32 + (lane & 3) * 8;
                        const uint32_t off = (m < a.M && n < a.N) ? ((uint32_t)m * (uint32_t)a.N + (uint32_t)n) * 2u : kOobOffset;
                        __builtin_amdgcn_raw_buffer_store_b128(v, rCst, (int)off, 0, 0);
                    }
                    asm volatile("" ::: "memory");
                    __builtin_amdgcn_sched_barrier(0);     // one 32x32 block at a time: keeps the accumulator copies few
                }
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0070);       // the loads issued past the last tile (all zeros) have landed too
}

// ======================================================================================================
// dW:  D[i][o] = sum_t X[t][i] * dY[t][o]   (M <-> i, N <-> o, K = T; both operand tiles KM)
// and, on the accumulators, for every weight (o, i):
//   Block-AP:  clamped = bit of the clamp plane; q = code; r = q - zbar
//              cs = clamped ? r : r - w/s ;  dW = clamped ? 0 : D ;  ds += D*cs ;  dz += clamped ? -s*D : 0
//   E2E-QP  :  ds += D * (q - z) ;  dz += -s*D  (dz only when asked for: zero points trained end to end)
// M <-> i puts the 32 columns of a group segment into the registers of one lane pair, so the group sums
// need one cross-lane exchange per 32x32 block.
// ======================================================================================================
struct GemmDwArgs {
    const bf16_t *X, *dY; const void *W; const uint32_t *codes; const uint8_t *clampbits; const floatx2 *sz;
    void *dW; float *ds, *dz, *part_ds, *part_dz;
    int T, I, O, G, g;
    uint32_t x_bytes, dy_bytes, w_bytes, codes_bytes, clamp_bytes, sz_bytes;
    int tiles_m, tiles_n;
    int direct;           // 1: every group lies inside one tile -> final ds/dz; 0: per-32-column partials
    SkPlan sk;            // which tiles, or parts of tiles, a workgroup computes (kernels that cut tiles along T)
};

// The epilogue of the Block-AP kernel reads W and writes dW through LDS.  In the accumulator layout a lane holds one
// weight ROW (out-feature) and four consecutive in-features per quad, so straight from the registers every load or
// store instruction would touch 32 different rows, 8 or 16 bytes of each.  Instead a wave moves the W rows it needs as
// whole 128- or 256-byte row pieces (16 bytes per lane, straight into LDS), picks its quads out of LDS, puts the dW
// quads back in their place and writes the rows out the way they came in.
// A unit = 32 rows x UB blocks of 32 in-features, RBY bytes per row; a wave owns two unit-sized LDS slots.  The 16-byte
// chunks of a row are XOR-swizzled with (row >> 1) so that the 32 lanes of a quad read (32 rows, same chunk) spread
// over all banks (two rows share a chunk position: the 2-way conflict of an 8-byte access by 32 lanes is the minimum).
template <typename WT, int MI> struct DwStage {
    static constexpr int kEB = (int)sizeof(WT);
    static constexpr int UB = (8 / kEB) < MI ? (8 / kEB) : MI;       // blocks per unit: rows of at most 256 bytes
    static constexpr int RBY = UB * 32 * kEB;                         // 128 or 256
    static constexpr int CPR = RBY / 16, RPI = 64 / CPR, NIU = 32 / RPI;   // chunks per row, rows per instruction, instructions
    static constexpr int UNIT_BYTES = 32 * RBY;
    static constexpr int UPJ = MI / UB;                               // units per 32-row block column of the wave
    static_assert(MI % UB == 0 && RBY <= 256 && UNIT_BYTES == NIU * 1024, "unit geometry");
    // byte offset (inside a slot) of chunk 0 of this lane's row, with the row's swizzle and the lane's half folded in:
    // the 16-byte chunk c (bf16: the 8-byte half h of it) is at  lane_base ^ (c * 16)
    static __device__ __forceinline__ uint32_t lane_base(int lane)
    {
        const uint32_t ol = (uint32_t)lane & 31u, h = (uint32_t)lane >> 5, xo = ((ol >> 1) & (uint32_t)(CPR - 1)) << 4;
        return kEB == 2 ? (ol * RBY + 8u * h) | xo : (ol * RBY) | (xo ^ (h << 4));
    }
    // chunk of quad q of block ii of the unit (for fp32 the lane's half is a chunk of its own, folded into lane_base)
    static constexpr uint32_t quad_chunk_bytes(int ii, int q) { return (uint32_t)(kEB == 2 ? ii * 4 + q : ii * 8 + 2 * q) * 16u; }
};

template <typename WT> struct WQuad;     // four consecutive weights of one row, to and from LDS
template <> struct WQuad<bf16_t> {
    static __device__ __forceinline__ void read(const unsigned char *p, float (&v)[4])
    {
        const uintx2 u = *reinterpret_cast<const uintx2 *>(p);
        v[0] = __uint_as_float(u[0] << 16); v[1] = __uint_as_float(u[0] & 0xFFFF0000u);
        v[2] = __uint_as_float(u[1] << 16); v[3] = __uint_as_float(u[1] & 0xFFFF0000u);
    }
    static __device__ __forceinline__ void write(unsigned char *p, const float (&d)[4])
    {
        floatx2 lo, hi;
        lo[0] = d[0]; lo[1] = d[1]; hi[0] = d[2]; hi[1] = d[3];
        const bf16x2 a = __builtin_convertvector(lo, bf16x2), b = __builtin_convertvector(hi, bf16x2);   // one packed convert each
        uintx2 o;
        o[0] = __builtin_bit_cast(uint32_t, a); o[1] = __builtin_bit_cast(uint32_t, b);
        *reinterpret_cast<uintx2 *>(p) = o;
    }
};
template <> struct WQuad<float> {
    static __device__ __forceinline__ void read(const unsigned char *p, float (&v)[4])
    {
        const floatx4 u = *reinterpret_cast<const floatx4 *>(p);
        v[0] = u[0]; v[1] = u[1]; v[2] = u[2]; v[3] = u[3];
    }
    static __device__ __forceinline__ void write(unsigned char *p, const float (&d)[4])
    {
        *reinterpret_cast<floatx4 *>(p) = floatx4{d[0], d[1], d[2], d[3]};
    }
};

// K-major tiles ([k][COLS] bf16, filled by direct-to-LDS loads of 1 KB = kmRowsPerLoad rows each): in the operand layout
// of the 16x16x32 MFMA the two groups of sixteen lanes that the LDS serves together read the same 32 bytes of columns
// eight rows apart, and rows of 256 or 512 bytes all start on the same bank, so the two groups collided on every read
// (SQ_LDS_BANK_CONFLICT: 45 M cycles per launch at the 7B shapes).  Every eight rows are therefore followed by a gap of 32
// bytes: the second group's pieces land in the other half of each 64-byte unit (counter back to what the epilogue
// leaves, 1.6 M).  Gaps of 128 or 256 bytes do not help (the banks repeat every 256 bytes and the swizzle of the 64-byte
// units already uses all four positions), and swapping the halves by a swizzle of the columns reorders the 16-byte
// chunks that four neighbouring lanes fetch from memory, which costs far more than the conflicts did (-19 %).
template <int COLS> constexpr int kmRowsPerLoad = 64 / (COLS / 8);
constexpr int kmGapElems = 16;
template <int COLS> __host__ __device__ constexpr int km_row_elems(int k) { return k * COLS + (k >> 3) * kmGapElems; }
template <int COLS> constexpr int kmTileElems(int rows) { return rows * COLS + (rows / 8) * kmGapElems; }

// LDS the dW kernel asks for: the K loop's tile ring, or (Block-AP) the epilogue's stage plus the group-sum partials.
template <typename WT, bool BLOCK_AP, int BM, int BN, int BK, int NS, int WGM, int WGN>
constexpr size_t dw_stage_bytes()
{
    return BLOCK_AP ? (size_t)WGM * WGN * 2 * DwStage<WT, BM / WGM / 32>::UNIT_BYTES : 0;
}
template <typename WT, bool BLOCK_AP, int BM, int BN, int BK, int NS, int WGM, int WGN>
constexpr size_t dw_smem_bytes()
{
    const size_t ring = (size_t)NS * (kmTileElems<BM>(BK) + kmTileElems<BN>(BK)) * sizeof(bf16_t);
    const size_t epi = dw_stage_bytes<WT, BLOCK_AP, BM, BN, BK, NS, WGM, WGN>() + (size_t)2 * (BM / 32) * BN * sizeof(float);
    return ring > epi ? ring : epi;
}

// ---- KM tile filled by direct-to-LDS loads ------------------------------------------------------------------
// Tile [BK][COLS] bf16, rows unpadded.  A transpose read touches four consecutive k rows, 64 bytes of each, so
// the 64-byte units of a row are XOR-swizzled with (k & 3) to spread those rows over the banks.
template <int COLS>
__device__ __forceinline__ int km_swz_col(int k, int col) { return (((col >> 5) ^ (k & 3)) << 5) | (col & 31); }

// A fragment of the tile as an operand of v_mfma_f32_16x16x32_bf16: the lane holds column col0 + lane % 16 and the eight
// k values 32 ks + 8 (lane / 16) + 0 .. 7.  Every group of 16 lanes reads a patch of 4 k rows x 16 columns per instruction
// (the transpose read hands lane i of the group four k-consecutive values of column i).
template <int COLS>
__device__ __forceinline__ bf16x8 frag_km16_swz(const bf16_t *tile, int col0, int ks, int lane)
{
    const int i = lane & 15, b = lane >> 4;
    const int k = ks * 32 + b * 8 + (i >> 2), col = col0 + (i & 3) * 4;
    const int c = km_swz_col<COLS>(k, col);                                               // (k + 4) & 3 == k & 3
    typedef short4v __attribute__((address_space(3))) * lds_p;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(tile + km_row_elems<COLS>(k) + c));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(tile + km_row_elems<COLS>(k + 4) + c));
    typedef short short8v __attribute__((ext_vector_type(8)));
    short8v r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// Streams consecutive [BK][COLS] row blocks of a row-major [rows][ld] bf16 matrix into LDS tiles, one direct-to-LDS
// instruction at a time (LOADS per wave and tile, RPI rows each).  Every instruction keeps its own running byte offset,
// so issuing one costs a scalar move to M0, the load and one add.  Columns past `ld` start at an out-of-range offset and
// advance like the others: tensors are smaller than 2 GiB, so 2 GiB plus any offset into one stays out of range (no
// wrap-around); rows past the end of the matrix fail the buffer's range check.
template <int BK, int COLS, int NW>
struct KmLoader {
    static constexpr int CPR = COLS / 8, RPI = kmRowsPerLoad<COLS>, LOADS = BK / RPI / NW;   // chunks per row, rows per instruction
    static_assert(BK % (RPI * NW) == 0 && CPR <= 64, "tile / wave mismatch");
    uint32_t off[LOADS], adv;                 // adv: bytes from one K tile to the next, the same for every lane
    __device__ __forceinline__ void init(int ld, int col0, int wave, int lane)
    {
#pragma unroll
        for (int it = 0; it < LOADS; ++it) {
            const int rb = (wave * LOADS + it) * RPI;                 // wave-uniform first row
            const int k = rb + lane / CPR, p = lane % CPR;
            const int col = col0 + (((p >> 2) ^ (k & 3)) << 5) + (p & 3) * 8;
            off[it] = col < ld ? ((uint32_t)k * (uint32_t)ld + (uint32_t)col) * 2u : kOobOffset;
        }
        adv = (uint32_t)BK * (uint32_t)ld * 2u;
    }
    // start n tiles further along K
    __device__ __forceinline__ void skip_tiles(int n)
    {
#pragma unroll
        for (int it = 0; it < LOADS; ++it) off[it] += (uint32_t)n * adv;
    }
    // instruction `it` of the next tile for this instruction slot; tile_lds = LDS address of the destination tile
    __device__ __forceinline__ void issue(const RawRsrc &r, int it, uint32_t tile_lds, int wave)
    {
        load_to_lds16_at(r, tile_lds + (uint32_t)(km_row_elems<COLS>((wave * LOADS + it) * RPI) * 2), off[it]);
        off[it] += adv;
    }
};

// s_waitcnt operand: "at most N vector-memory operations still outstanding, all LDS operations complete".
constexpr int waitcnt_vm_lgkm0(int n) { return (n & 15) | 0x70 | ((n >> 4) << 14); }

// CUT: the grid is as large as the chip holds at once and a workgroup works through the items that a.sk deals it: whole
// tiles, and parts (along T) of tiles that it shares with others (see SkPlan; the accumulators of the parts meet in
// sk_hand_in, and the contributor that ends up with their sum runs the tile's epilogue).  Otherwise one tile per workgroup.
template <int BITS, typename WT, bool BLOCK_AP, int BM, int BN, int BK, int NS, int WGM, int WGN, bool CUT>
__global__ __launch_bounds__(64 * WGM * WGN) void k_gemm_dw(const GemmDwArgs a)
{
    constexpr int NT = 64 * WGM * WGN, NW = WGM * WGN, WTM = BM / WGM, WTN = BN / WGN, MI = WTM / 32, NI = WTN / 32;
    constexpr int A_ELEMS = kmTileElems<BM>(BK), B_ELEMS = kmTileElems<BN>(BK);      // with the gaps between the 1 KB pieces
    static_assert(NS >= 2, "at least two LDS stages");
    static_assert(NS * (A_ELEMS + B_ELEMS) * 2 >= 2 * (BM / 32) * BN * 4, "partials must fit in the tile buffers");

    want_agpr_accumulators<MI * NI * 16>();
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t *sA = reinterpret_cast<bf16_t *>(smem_raw);            // [NS][A_ELEMS]
    bf16_t *sB = sA + NS * A_ELEMS;                               // [NS][B_ELEMS]

    int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave / WGN, wn = wave % WGN;
    const RawRsrc rX = make_raw_rsrc(a.X, a.x_bytes);
    const RawRsrc rY = make_raw_rsrc(a.dY, a.dy_bytes);
    const uint32_t ldsA = lds_addr_of(sA), ldsB = lds_addr_of(sB);

  for ([[maybe_unused]] int item = 0;; ++item) {
    // What depends on the lane alone would otherwise be worked out once, in front of this loop, and kept in registers
    // through every phase of every item; the main loop has none to spare.
    if constexpr (CUT) asm volatile("" : "+v"(tid));
    int lane = tid & 63;
    int tm, tn;
    [[maybe_unused]] SkItem si;
    if constexpr (CUT) {
        if (!sk_item(a.sk, a.tiles_m * a.tiles_n, a.tiles_m, a.tiles_n, 8, item, si)) break;
        tm = si.tm; tn = si.tn;
    } else {
        tile_of_block(a.tiles_m, a.tiles_n, tm, tn);
    }
    const int m0 = tm * BM, n0 = tn * BN;      // m0: first in-feature i, n0: first out-feature o
    // K tiles (of BK tokens) of this item: all of them, or the pairs [kb, ke) of a part (an even number of tiles, except
    // that the last pair of all may lack its second tile)
    int kt0 = 0, nk = (a.T + BK - 1) / BK;
    if constexpr (CUT) {
        kt0 = 2 * si.kb;
        nk = (2 * si.ke < nk ? 2 * si.ke : nk) - kt0;
    }
    KmLoader<BK, BM, NW> ldX;
    KmLoader<BK, BN, NW> ldY;
    ldX.init((int)a.I, m0, wave, lane);
    ldY.init((int)a.O, n0, wave, lane);
    if constexpr (CUT) { ldX.skip_tiles(kt0); ldY.skip_tiles(kt0); }
    constexpr int LA = KmLoader<BK, BM, NW>::LOADS, LB = KmLoader<BK, BN, NW>::LOADS, ND = LA + LB;
    // load number d (0 .. ND-1) of the NEXT K tile (tiles are fetched strictly in order) into LDS buffer `buf`
    auto issue_load = [&](int d, int buf) {
        if (d < LA) ldX.issue(rX, d, ldsA + (uint32_t)(buf * A_ELEMS * 2), wave);
        else ldY.issue(rY, d - LA, ldsB + (uint32_t)(buf * B_ELEMS * 2), wave);
    };
    auto load_tiles = [&](int buf) {
#pragma unroll
        for (int d = 0; d < ND; ++d) issue_load(d, buf);
    };

    floatx4 acc[MI][NI][4];      // [q] = registers 4 q .. 4 q + 3 of the block
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r >> 2][r & 3] = 0.0f;

    // The contraction runs on v_mfma_f32_16x16x32_bf16 (measured 4-7 % ahead of the 32x32x16 form in this loop, which
    // moves twice the accumulator registers per flop): the 32 x 32 block (i, j) of the wave is four 16 x 16 products, and
    // product (ii, jj) lives in acc[i][j][2 ii + jj] until the end of the K loop, where the blocks
    // are brought into the lane order of the 32 x 32 form that the epilogue is written for (see the start of the epilogue).
    // A K tile is KS slices of 32.  Per slice a wave needs MA = 2 MI fragments of X and NB = 2 NI of dY (4 registers
    // each).  The dY fragments are double-buffered; an X fragment is used by NB consecutive MFMAs only, so the fragment
    // of the next slice takes its registers as soon as those have been issued.
    constexpr int KS = BK / 32, MA = 2 * MI, NB = 2 * NI;
    static_assert(BK % 32 == 0 && KS >= 2 && MA >= NB, "slices of 32, at least two per tile; B fragments ride along with the first A fragments");
    bf16x8 fa[MA], fb[2][NB];
    auto frag_a = [&](int buf, int ks, int ia) { return frag_km16_swz<BM>(sA + buf * A_ELEMS, wm * WTM + ia * 16, ks, lane); };
    auto frag_b = [&](int buf, int ks, int jb) { return frag_km16_swz<BN>(sB + buf * B_ELEMS, wn * WTN + jb * 16, ks, lane); };
    auto mfma16 = [&](auto ia_, auto jb_, int pb) __attribute__((always_inline)) {
        constexpr int ia = decltype(ia_)::value, jb = decltype(jb_)::value;
        floatx4 &c = acc[ia >> 1][jb >> 1][(ia & 1) * 2 + (jb & 1)];
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[ia], fb[pb][jb], c, 0, 0, 0);
    };
    // One K tile.  Same pipeline as the forward kernel: the barrier sits before the last slice, whose MFMAs then cover
    // the first fragment reads of the next tile and the issue of the loads for a later tile.  The K tiles go round a ring
    // of NS LDS stages: behind the barrier of tile kt the stage of tile kt itself is free (its last fragments are in
    // registers) and takes tile kt + NS, so a load has NS - 1 tile times to land; the barrier waits only for the loads
    // of tile kt + 1 (vector-memory operations complete in order: "all but the newest (NS - 2) batches").
    // P = dY fragment buffer that holds slice 0 of this tile; slices alternate, so the next tile starts in (P + KS) & 1.
    auto step = [&](auto par, int buf, int nxt) __attribute__((always_inline)) {
        constexpr int P = decltype(par)::value;
        // MFMAs of X fragment ia, then, in their shadow, the fragments that replace it (and one dY fragment of the next
        // slice), from slice `ks_next` of stage `src`; in the last slice also one or two loads for tile kt + NS.
        auto run_slice = [&](auto pb_, auto last_, int src, int ks_next) __attribute__((always_inline)) {
            constexpr int pb = decltype(pb_)::value;
            constexpr bool last = decltype(last_)::value;
            static_for<MA>([&](auto ia_) __attribute__((always_inline)) {
                constexpr int ia = decltype(ia_)::value;
                static_for<NB>([&](auto jb_) __attribute__((always_inline)) { mfma16(ia_, jb_, pb); });
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (last) {
#pragma unroll
                    for (int d = 0; d < ND; ++d)
                        if (d * MA / ND == ia) issue_load(d, buf);
                }
                fa[ia] = frag_a(src, ks_next, ia);
                if constexpr (ia < NB) fb[pb ^ 1][ia] = frag_b(src, ks_next, ia);
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        static_for<KS - 1>([&](auto ks_) __attribute__((always_inline)) {
            constexpr int ks = decltype(ks_)::value;
            run_slice(IC<((P + ks) & 1)>{}, IC<0>{}, buf, ks + 1);
        });
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NS - 2) * ND));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        run_slice(IC<((P + KS - 1) & 1)>{}, IC<1>{}, nxt, 0);
    };

    if (nk > 0) {
#pragma unroll
        for (int st = 0; st < NS; ++st) load_tiles(st);            // tiles 0 .. NS-1 (past T: zeros)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NS - 1) * ND));      // tile 0 has landed
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) fb[0][jb] = frag_b(0, 0, jb);
#pragma unroll
        for (int ia = 0; ia < MA; ++ia) fa[ia] = frag_a(0, 0, ia);
        // Two tiles per trip, so that the fragment buffers alternate at compile time when a tile has an odd number of
        // slices; with an odd tile count the extra tile lies past T and multiplies zeros.
        int buf = 0;
        for (int kt = 0; kt < nk; kt += 2) {
            int nxt = buf + 1 == NS ? 0 : buf + 1;
            step(IC<0>{}, buf, nxt);
            buf = nxt; nxt = buf + 1 == NS ? 0 : buf + 1;
            step(IC<(KS & 1)>{}, buf, nxt);
            buf = nxt;
        }
    }
    wait_all_and_barrier();   // tile buffers become the partial-sum arrays
    if constexpr (CUT) {
        // a tile cut along T: only the contributor that ends up with the sum of all parts goes on to the epilogue
        asm volatile("" : "+v"(tid));
        if (si.parts > 1 && !sk_hand_in<MI, NI, NT, 4>(a.sk, si, acc, tid)) continue;      // nothing else is alive here: four blocks at a time
    }
    // what the epilogue derives from the lane is worked out here, not in front of the K loop (see the top of the loop)
    asm volatile("" : "+v"(tid));
    lane = tid & 63;

    // ---- epilogue ----------------------------------------------------------------------------------
    using SG = DwStage<WT, MI>;
    constexpr uint32_t kStageBytes = (uint32_t)dw_stage_bytes<WT, BLOCK_AP, BM, BN, BK, NS, WGM, WGN>();
    float *p_ds = reinterpret_cast<float *>(smem_raw + kStageBytes);      // [BM/32][BN]
    float *p_dz = p_ds + (BM / 32) * BN;
    const __amdgpu_buffer_rsrc_t rC = make_rsrc(a.codes, a.codes_bytes);
    const __amdgpu_buffer_rsrc_t rS = make_rsrc(a.sz, a.sz_bytes);
    const __amdgpu_buffer_rsrc_t rB = make_rsrc(a.clampbits, a.clamp_bytes);
    const __amdgpu_buffer_rsrc_t rDW = make_rsrc(a.dW, a.dW != nullptr ? a.w_bytes : 0u);    // no dW wanted: stores dropped
    const RawRsrc rWraw = make_raw_rsrc(a.W, a.w_bytes);
    const uint32_t code_row_bytes = (uint32_t)a.I / 32u * (4u * WorkCodes<BITS>::kWords);
    const int h = lane >> 5;
    const int ibw = m0 + wm * WTM;                             // first in-feature of this wave

    // What a lane needs of its weight row for the MI blocks of one block column j, fetched with few, wide loads: the
    // codes and the clamp bits of the MI blocks lie side by side in memory.  (Blocks past the end of a row read what
    // follows, or zeros past the buffer; their accumulators and their W are zero, so whatever the codes are the sums
    // come out as zero, and nothing of such a block is stored.)
    constexpr int CODE_WORDS = MI * WorkCodes<BITS>::kWords, CODE_LOADS = (CODE_WORDS + 3) / 4;
    struct RowOps { uint32_t cw[CODE_LOADS * 4]; intx2 sv[MI]; uint32_t ncl[MI]; };
    auto load_row_ops = [&](int j, RowOps &r) {
        const int o = n0 + wn * WTN + j * 32 + (lane & 31);
        const bool row_ok = o < a.O && ibw < a.I;
        const uint32_t c0 = (uint32_t)o * code_row_bytes + (uint32_t)(ibw >> 5) * (4u * WorkCodes<BITS>::kWords);
#pragma unroll
        for (int q = 0; q < CODE_LOADS; ++q) {
            if constexpr (CODE_WORDS % 4 == 0) {
                const intx4 v = buf_load16(rC, row_ok ? c0 + 16u * q : kOobOffset);
                r.cw[4 * q] = v[0]; r.cw[4 * q + 1] = v[1]; r.cw[4 * q + 2] = v[2]; r.cw[4 * q + 3] = v[3];
            } else {
                static_assert(CODE_WORDS % 4 == 0 || CODE_WORDS == 2, "code words per wave row");
                const intx2 v = buf_load8(rC, row_ok ? c0 : kOobOffset);
                r.cw[0] = v[0]; r.cw[1] = v[1]; r.cw[2] = 0u; r.cw[3] = 0u;
            }
        }
        if constexpr (BLOCK_AP) {
            const uint32_t b0 = (uint32_t)o * (uint32_t)(a.I >> 3) + (uint32_t)(ibw >> 3);
            if constexpr (MI == 4) {
                const intx4 v = buf_load16(rB, row_ok ? b0 : kOobOffset);
                r.ncl[0] = v[0]; r.ncl[1] = v[1]; r.ncl[2] = v[2]; r.ncl[3] = v[3];
            } else if constexpr (MI == 2) {
                const intx2 v = buf_load8(rB, row_ok ? b0 : kOobOffset);
                r.ncl[0] = v[0]; r.ncl[1] = v[1];
            } else {
#pragma unroll
                for (int i = 0; i < MI; ++i) r.ncl[i] = (uint32_t)buf_load4(rB, row_ok ? b0 + 4u * i : kOobOffset);
            }
        }
        // (s, zbar) of each block's group: one load per group the wave's blocks touch (wave-uniform branches)
        int grp_prev = -1;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int ib = ibw + i * 32, grp = ib < a.I ? ib / a.g : -1 - i;
            if (i > 0 && grp == grp_prev) r.sv[i] = r.sv[i - 1];
            else r.sv[i] = buf_load8(rS, (o < a.O && ib < a.I) ? ((uint32_t)o * (uint32_t)a.G + (uint32_t)grp) * 8u : kOobOffset);
            grp_prev = grp;
        }
    };

    // W rows of unit u = (j, v): global byte offset of this lane's 16-byte chunk, per instruction
    auto unit_offsets = [&](int u, uint32_t (&off)[SG::NIU]) {
        const int j = u / SG::UPJ, v = u % SG::UPJ;
#pragma unroll
        for (int k = 0; k < SG::NIU; ++k) {
            const int r = k * SG::RPI + lane / SG::CPR, c = (lane % SG::CPR) ^ ((r >> 1) & (SG::CPR - 1));
            const int o = n0 + wn * WTN + j * 32 + r, i0 = ibw + v * SG::UB * 32 + c * (16 / SG::kEB);
            off[k] = (o < a.O && i0 < a.I) ? ((uint32_t)o * (uint32_t)a.I + (uint32_t)i0) * (uint32_t)SG::kEB : kOobOffset;
        }
    };
    const uint32_t stage_lds = lds_addr_of(smem_raw);
    auto slot_bytes = [&](int slot) { return (uint32_t)((wave * 2 + slot) * SG::UNIT_BYTES); };
    auto issue_unit = [&](int slot, const uint32_t (&off)[SG::NIU]) {
#pragma unroll
        for (int k = 0; k < SG::NIU; ++k) load_to_lds16_at(rWraw, stage_lds + slot_bytes(slot) + (uint32_t)(k * 1024), off[k]);
    };

    constexpr int NU = BLOCK_AP ? NI * SG::UPJ : 0;
    uint32_t goff[2][SG::NIU];
    if constexpr (BLOCK_AP) {
        // the first unit starts to stream in at once; the second follows below, a later one when its slot has been written out
        unit_offsets(0, goff[0]);
        issue_unit(0, goff[0]);
    }
    RowOps rops[2];
    load_row_ops(0, rops[0]);

    // ---- accumulators into the lane order of the 32 x 32 MFMA (while the loads above are under way) ----------------
    // From the K loop a lane holds, of block (i, j), product (ii, jj) in registers 4 (2 ii + jj) + b: row 16 ii +
    // 4 (lane / 16) + b, column 16 jj + lane % 16.  What follows wants register 4 q + b to be row 8 q + 4 (lane / 32) + b
    // of column lane % 32.  Rows 16 ii .. 16 ii + 15 are quads q = 2 ii and 2 ii + 1, so each half of a block is
    // converted by itself: every lane puts its two quads (16 bytes each) into a 2 KB patch of LDS that belongs to its
    // wave, [column][row quad] with the quad's place rotated by column / 4 against bank conflicts, and takes the two
    // quads it owns in the other order.  LDS accesses of a wave complete in order; nothing else touches the patch.
    {
        // Block-AP: the wave's second W slot, which is still empty; else the tile ring behind the partial sums
        const uint32_t patch = BLOCK_AP ? slot_bytes(1) : (uint32_t)(2 * (BM / 32) * BN * sizeof(float)) + (uint32_t)(wave * 2048);
        static_assert(BLOCK_AP ? SG::UNIT_BYTES >= 2048 : NS * (A_ELEMS + B_ELEMS) * 2 >= 2 * (BM / 32) * BN * 4 + NW * 2048, "room for the patch");
        const int c16 = lane & 15, rq_in = lane >> 4, c32 = lane & 31, h32 = lane >> 5;
        uint32_t at_in[2], at_out[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int col = 16 * t + c16, rq = 2 * t + h32;
            at_in[t] = patch + (uint32_t)(col * 64 + ((rq_in + (col >> 2)) & 3) * 16);
            at_out[t] = patch + (uint32_t)(c32 * 64 + ((rq + (c32 >> 2)) & 3) * 16);
        }
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        *reinterpret_cast<floatx4 *>(smem_raw + at_in[t]) = acc[i][j][2 * hh + t];
                    }
                    asm volatile("" ::: "memory");
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        acc[i][j][2 * hh + t] = *reinterpret_cast<const floatx4 *>(smem_raw + at_out[t]);
                    }
                    asm volatile("" ::: "memory");
                    __builtin_amdgcn_wave_barrier();
                }
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);            // lgkmcnt(0): the patch has been read out, its place may take W rows
    asm volatile("" ::: "memory");
    if constexpr (NU > 1) {
        unit_offsets(1, goff[1]);
        issue_unit(1, goff[1]);
    }
    // The compiler does not see the loads into LDS: wait for them here.  The second unit was requested last and may
    // still be under way; its block column waits for it below.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(NU > 1 ? SG::NIU : 0));
    asm volatile("" ::: "memory");
    const uint32_t lane_base = SG::lane_base(lane);

#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int ol = wn * WTN + j * 32 + (lane & 31), o = n0 + ol;
        if (j + 1 < NI) load_row_ops(j + 1, rops[(j + 1) & 1]);      // under this column's arithmetic
        const RowOps &ro = rops[j & 1];
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int ib = ibw + i * 32;                           // first of 32 in-features; whole block valid or not
            const bool valid = (o < a.O) && (ib < a.I);
            [[maybe_unused]] const int u = j * SG::UPJ + i / SG::UB, ii = i % SG::UB, slot = u & 1;
            if constexpr (BLOCK_AP) {
                if (ii == 0 && u >= 1) {       // requested after the first unit, or when its slot became free (below)
                    asm volatile("" ::: "memory");
                    __builtin_amdgcn_s_waitcnt(0x0070);
                    asm volatile("" ::: "memory");
                }
            }
            WorkCodes<BITS> cw;
#pragma unroll
            for (int k = 0; k < WorkCodes<BITS>::kWords; ++k) cw.w[k] = ro.cw[i * WorkCodes<BITS>::kWords + k];
            // this lane owns codes 8a + 4h + b (a, b in 0..3): four consecutive codes per a, h fields further along
            const uint32_t pre = (uint32_t)h * WorkCodes<BITS>::kField;
            uint32_t cq[4] = {cw.four(0, pre), cw.four(8, pre), cw.four(16, pre), cw.four(24, pre)};
            // keep the four masked words as they are: folded into one bit-field extract per code, the byte-to-float
            // conversions (v_cvt_f32_ubyte0..3, one instruction per code) would each need an extract in front
#pragma unroll
            for (int q = 0; q < 4; ++q) asm volatile("" : "+v"(cq[q]));
            const float s = __int_as_float(ro.sv[i][0]), zb = __int_as_float(ro.sv[i][1]);
            float sum_s = 0.0f, sum_z = 0.0f;
            if constexpr (BLOCK_AP) {
                // keep-bits: 1 where Eq.(1) did NOT clamp the weight
                const uint32_t ncl = ~(ro.ncl[i] >> (4 * h));
                const float rinv = valid ? 1.0f / s : 0.0f;
                const uint32_t quads = slot_bytes(slot) + lane_base;       // chunk bits are clear in slot_bytes
                // Per weight, with keep = all ones where it was not clamped (one bit-field extract) and bitwise ANDs
                // in place of selects:  du = D & keep (this is dW),  cs = (q - (w & keep) / s) - zbar, which is
                // r - w/s in range and r = q - zbar where clamped,  sum over clamped D = sum D - sum du.
                float sum_d = 0.0f, sum_u = 0.0f;
#define EQAT_ELEM(Q, B)                                                                                   \
    {                                                                                                     \
        const float d = acc[i][j][Q][B];                                                         \
        const uint32_t keep = (uint32_t)((int32_t)(ncl << (31 - ((Q) * 8 + (B)))) >> 31);                 \
        const float du = __uint_as_float(__float_as_uint(d) & keep);                                      \
        const float wm = __uint_as_float(__float_as_uint(wv[B]) & keep);                                  \
        const float cs = __builtin_fmaf(-wm, rinv, byte_to_float(cq[Q], B)) - zb;                         \
        sum_s = __builtin_fmaf(d, cs, sum_s);                                                             \
        sum_d += d;                                                                                       \
        sum_u += du;                                                                                      \
        dwv[B] = du;                                                                                      \
    }
#define EQAT_QUAD(Q)                                                                                      \
    {                                                                                                     \
        unsigned char *const cell = smem_raw + (quads ^ SG::quad_chunk_bytes(ii, (Q)));                   \
        float wv[4], dwv[4];                                                                              \
        WQuad<WT>::read(cell, wv);                                                                        \
        EQAT_ELEM(Q, 0) EQAT_ELEM(Q, 1) EQAT_ELEM(Q, 2) EQAT_ELEM(Q, 3)                                   \
        WQuad<WT>::write(cell, dwv);                                                                      \
    }
                EQAT_QUAD(0) EQAT_QUAD(1) EQAT_QUAD(2) EQAT_QUAD(3)
#undef EQAT_QUAD
#undef EQAT_ELEM
                sum_z = sum_d - sum_u;
            } else {
#define EQAT_ELEM(Q, B)                                                                                   \
    {                                                                                                     \
        const float d = acc[i][j][Q][B];                                                         \
        sum_s = __builtin_fmaf(d, byte_to_float(cq[Q], B) - zb, sum_s);                                   \
        sum_z += d;                                                                                       \
    }
#define EQAT_QUAD(Q) EQAT_ELEM(Q, 0) EQAT_ELEM(Q, 1) EQAT_ELEM(Q, 2) EQAT_ELEM(Q, 3)
                EQAT_QUAD(0) EQAT_QUAD(1) EQAT_QUAD(2) EQAT_QUAD(3)
#undef EQAT_QUAD
#undef EQAT_ELEM
            }
            sum_s += __shfl_xor(sum_s, 32);
            sum_z += __shfl_xor(sum_z, 32);
            if (h == 0) {
                p_ds[(wm * MI + i) * BN + ol] = sum_s;
                p_dz[(wm * MI + i) * BN + ol] = sum_z;
            }
            if constexpr (BLOCK_AP) {
                if (ii == SG::UB - 1) {
                    // The unit is complete: dW sits where W sat.  Rows go out the way they came in.  LDS accesses of a
                    // wave complete in order, so the reads below see the quads every lane of the wave has written.
                    asm volatile("" ::: "memory");
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int k = 0; k < SG::NIU; ++k) {
                        const intx4 v = *reinterpret_cast<const intx4 *>(smem_raw + slot_bytes(slot) + (uint32_t)(k * 1024 + lane * 16));
                        __builtin_amdgcn_raw_buffer_store_b128(v, rDW, (int)goff[slot][k], 0, 0);
                    }
                    if (u + 2 < NU) {
                        asm volatile("" ::: "memory");
                        __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): the slot has been read out
                        asm volatile("" ::: "memory");
                        unit_offsets(u + 2, goff[slot]);
                        issue_unit(slot, goff[slot]);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);     // one 32x32 block at a time
        }
    }
    __syncthreads();
    if (a.direct) {
        // every group of this tile's rows is complete here: sum its g/32 block partials in order
        const int bpg = a.g >> 5, gpt = BM / a.g;
        for (int e = tid; e < gpt * BN; e += NT) {
            const int ol = e % BN, gi = e / BN, o = n0 + ol, i0 = m0 + gi * a.g;
            if (o >= a.O || i0 >= a.I) continue;
            float vs = 0.0f, vz = 0.0f;
            for (int k = 0; k < bpg; ++k) {
                vs += p_ds[(gi * bpg + k) * BN + ol];
                vz += p_dz[(gi * bpg + k) * BN + ol];
            }
            const size_t gidx = (size_t)o * a.G + i0 / a.g;
            if (a.ds != nullptr) a.ds[gidx] = vs;
            if (a.dz != nullptr) a.dz[gidx] = -a.sz[gidx][0] * vz;
        }
    } else {
        const int nb32 = a.I >> 5;
        for (int e = tid; e < (BM / 32) * BN; e += NT) {
            const int ol = e % BN, blk = e / BN, o = n0 + ol, i0 = m0 + blk * 32;
            if (o >= a.O || i0 >= a.I) continue;
            a.part_ds[(size_t)o * nb32 + (i0 >> 5)] = p_ds[blk * BN + ol];
            if (a.dz != nullptr) a.part_dz[(size_t)o * nb32 + (i0 >> 5)] = p_dz[blk * BN + ol];
        }
    }
    if constexpr (!CUT) break;
    __syncthreads();          // the next item's tiles go where the sums were
  }
}

// ======================================================================================================
// host side
// ======================================================================================================
namespace {

template <int BM_, int BN_, int BK_, int WGM_, int WGN_> struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_;
};
typedef Tile<128, 128, 64, 2, 2> TileSmall;   // 4 waves, 64x64 per wave: problems with few big tiles
typedef Tile<256, 256, 64, 2, 4> TileBig;     // 8 waves, 128x64 per wave
// dW: same output tiles.  The kernel takes any number of LDS stages NS and any K-tile width; measured, two stages of 64
// win: the big tile fits three stages only with 48-wide K tiles (3 x 48 KB), whose extra barriers cost what the deeper
// prefetch gains (-1 %); the small tile with three stages (96 KB) loses the second workgroup per CU (-17 %).
template <int BM_, int BN_, int BK_, int NS_, int WGM_, int WGN_> struct DwTile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, NS = NS_, WGM = WGM_, WGN = WGN_;
};
typedef DwTile<128, 128, 64, 2, 2, 2> DwTileSmall;
typedef DwTile<256, 256, 64, 2, 2, 4> DwTileBig;
static_assert(DwTileSmall::BM == TileSmall::BM && DwTileBig::BM == TileBig::BM, "group-fits-in-tile tests use Tile*::BM");

// the big tile unless it would leave a large part of the 256 CUs without a workgroup
bool use_small_tile(int64_t m, int64_t n)
{
    return ((m + 255) / 256) * ((n + 255) / 256) < 160;
}

// The kernels need more dynamic LDS than the default limit; the attribute is per kernel AND per device, so it is set
// once for every (instantiation, device) pair.  `done` is the caller's static mask of devices already served.
template <typename K> void allow_dynamic_lds(K kern, size_t smem, uint64_t &done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) dev = 0;
    if ((done >> dev) & 1u) return;
    (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    done |= (uint64_t)1 << dev;
}

// Workgroups of `smem` bytes of LDS that the device runs at the same time (LDS is what limits these kernels), rounded
// down to a multiple of 8.
constexpr int kMaxCus = 256;            // compute units of an MI355X; the workspace is sized for this many
constexpr int kSkCounterWords = 2 * 2 * 2 * kMaxCus;  // 2 G arrival counters and 2 G flags, G <= 2 workgroups per compute unit
int resident_workgroups(size_t smem)
{
    static int cus_of[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) dev = 0;
    if (cus_of[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = kMaxCus;
        cus_of[dev] = n < kMaxCus ? n : kMaxCus;
    }
    const int per_cu = smem * 2 <= 160 * 1024 ? 2 : 1;
    return (cus_of[dev] * per_cu) & ~7;
}

// How `resident` workgroups share `ntiles` tiles of `pairs` K-tile pairs each (see SkPlan).  One workgroup per tile
// when they all fit; otherwise whole tiles, except that (K long enough)
//   - between one and two rounds of tiles, with more than half a round beyond the first, every tile is cut along K into
//     equal runs (with more rounds, cutting the last 1.x of them into runs measured slower than leaving the last round
//     partly filled: 7B gate, 5.4 rounds: -3 %; 13B gate, 3.4 rounds: -4 %);
//   - with at most half a round of tiles beyond the whole rounds, those few tiles are split among groups of workgroups.
SkPlan plan_tiles(int ntiles, int pairs, int resident, float *partials, uint32_t *counters, bool runs = true)
{
    SkPlan sk{};
    sk.pairs = pairs; sk.partials = partials; sk.counters = counters;
    if (ntiles <= resident) return sk;                       // walk = 0
    sk.walk = 1;
    const int W = resident / 8, per = ntiles / 8, full = per / W;
    const bool even = (per % W == 0) && (ntiles % 8 == 0);
    const bool may_cut = !even && pairs >= 4 && partials != nullptr && counters != nullptr;
    sk.dp_rounds = (may_cut && runs && full == 1) ? 0 : (per + (ntiles % 8 ? 1 : 0) + W - 1) / W;
    // Few tiles beyond the whole rounds (at most half a round on every XCD): whole tiles first, then the rest split.
    // The tile arithmetic promises (1 - 1/c) of a round; measured, 5.4 rounds (7B gate, up) gain 2.6 %, 3.4 rounds (13B
    // gate) 1.5-2.3 %: the partly filled round that the split replaces ran at a higher clock, and the instantiation that
    // can cut is 1-5 % slower in its main loop.  Beyond six whole rounds the promise is smaller than that price.
    const int n_sk_max = per + (ntiles % 8 ? 1 : 0) - full * W;
    if (may_cut && full <= 6 && n_sk_max >= 1 && 2 * n_sk_max <= W && pairs >= 2 * kSkMaxSplit) { sk.dp_rounds = full; sk.split = 1; }
    return sk;
}

// Geometry of a fwd / dX launch: tiles, the XCD band, who computes what (SkPlan), the grid, and which instantiation runs.
struct QLaunchPlan { int tiles_m, tiles_n, band, ntiles, grid; SkPlan sk; bool cut_inst; };
template <bool BT, typename TS> constexpr size_t q_smem_bytes()
{
    constexpr int LDB = BT ? TS::BN + kPadKM : TS::BK + kPadKC;
    return 2 * (size_t)(TS::BM * TS::BK + (BT ? TS::BK * LDB : TS::BN * LDB)) * sizeof(bf16_t) + (size_t)TS::WGM * TS::WGN * kStoreStageBytes;
}
template <bool BT, typename TS>
QLaunchPlan plan_q(int M, int N, int K, float *partials, uint32_t *counters)
{
    QLaunchPlan q{};
    q.tiles_m = (M + TS::BM - 1) / TS::BM;
    q.tiles_n = (N + TS::BN - 1) / TS::BN;
    // Tile rows that one XCD walks together.  The activation panel of a tile row is eight times heavier than the code
    // panel of a tile column, so the 32 tiles an XCD holds at a time should span few rows and many columns (per K step
    // it fetches rows x 32 KB + columns x 6 KB: 4 rows x 8 columns 176 KB, 8 x 4 280 KB), and with an eighth of the tile
    // rows per band every XCD owns its rows outright, so that an activation panel is fetched by one XCD only.  Measured:
    // 4 (8192 tokens) and 2 (4096 tokens) are up to 2-4 % ahead of 8; 16 is 3 % behind.
    q.band = std::max(2, std::min(8, q.tiles_m / 8));
    // At most as many workgroups as the chip holds at once; with more tiles than that every workgroup walks several
    // (grid a multiple of 8, one share per XCD).
    q.ntiles = q.tiles_m * q.tiles_n;
    const int resident = resident_workgroups(q_smem_bytes<BT, TS>());
    q.sk = plan_tiles(q.ntiles, ((K + TS::BK - 1) / TS::BK + 1) / 2, resident, partials, counters);
    q.grid = q.sk.walk ? resident : q.ntiles;
    q.cut_inst = (q.sk.walk && (q.sk.dp_rounds == 0 || q.sk.split)) || K % (2 * TS::BK) != 0;
    return q;
}

template <int BITS, bool BT, typename TS>
void launch_q(const GemmQArgs &args, hipStream_t st)
{
    constexpr size_t smem = q_smem_bytes<BT, TS>();
    static_assert(smem + 64 <= 160 * 1024, "LDS of one CU");
    GemmQArgs a = args;
    a.c_bytes = (uint32_t)((size_t)a.M * a.N * 2);
    const QLaunchPlan q = plan_q<BT, TS>(a.M, a.N, a.K, a.sk.partials, a.sk.counters);
    a.tiles_m = q.tiles_m; a.tiles_n = q.tiles_n; a.band = q.band; a.sk = q.sk;
    const dim3 grid(q.grid), block(64 * TS::WGM * TS::WGN);
    if (q.cut_inst) {
        auto kern = k_gemm_q<BITS, BT, true, TS::BM, TS::BN, TS::BK, TS::WGM, TS::WGN>;
        static uint64_t attr_done = 0;
        allow_dynamic_lds(kern, smem, attr_done);
        kern<<<grid, block, smem, st>>>(a);
    } else {
        auto kern = k_gemm_q<BITS, BT, false, TS::BM, TS::BN, TS::BK, TS::WGM, TS::WGN>;
        static uint64_t attr_done = 0;
        allow_dynamic_lds(kern, smem, attr_done);
        kern<<<grid, block, smem, st>>>(a);
    }
}

template <bool BT>
void launch_q_bits(int bits, const GemmQArgs &a, hipStream_t st)
{
    const bool small = use_small_tile(a.M, a.N);
#define EQAT_GO(B) do { if (small) launch_q<B, BT, TileSmall>(a, st); else launch_q<B, BT, TileBig>(a, st); } while (0)
    if (bits == 2) EQAT_GO(2); else if (bits == 3) EQAT_GO(3); else EQAT_GO(4);
#undef EQAT_GO
}

// Geometry of a dW launch: tiles (rows: in-features, columns: out-features), and whether tiles are cut along T (then the
// grid is what the chip holds at once and sk says who computes what), or every tile has a workgroup of its own.
struct DwLaunchPlan { int tiles_m, tiles_n, ntiles, grid; SkPlan sk; bool cut; };
template <typename WT, bool AP, typename TS>
DwLaunchPlan plan_dw(int I, int O, int T, float *partials, uint32_t *counters)
{
    DwLaunchPlan d{};
    d.tiles_m = (I + TS::BM - 1) / TS::BM;
    d.tiles_n = (O + TS::BN - 1) / TS::BN;
    d.ntiles = d.tiles_m * d.tiles_n;
    const int resident = resident_workgroups(dw_smem_bytes<WT, AP, TS::BM, TS::BN, TS::BK, TS::NS, TS::WGM, TS::WGN>());
    d.sk = plan_tiles(d.ntiles, ((T + TS::BK - 1) / TS::BK + 1) / 2, resident, partials, counters, false);
    d.cut = d.sk.walk && (d.sk.dp_rounds == 0 || d.sk.split);
    if (!d.cut) d.sk = SkPlan{};
    d.grid = d.cut ? resident : d.ntiles;
    return d;
}

template <int BITS, typename WT, bool AP, typename TS>
void launch_dw_t(const GemmDwArgs &args, const SkScratch &scratch, hipStream_t st)
{
    constexpr size_t smem = dw_smem_bytes<WT, AP, TS::BM, TS::BN, TS::BK, TS::NS, TS::WGM, TS::WGN>();
    static_assert(smem + 64 <= 160 * 1024, "LDS of one CU");
    GemmDwArgs a = args;
    const DwLaunchPlan d = plan_dw<WT, AP, TS>(a.I, a.O, a.T, scratch.partials, scratch.counters);
    a.tiles_m = d.tiles_m;
    a.tiles_n = d.tiles_n;
    a.direct = (TS::BM % a.g == 0) ? 1 : 0;
    a.sk = d.sk;
    const dim3 grid(d.grid), block(64 * TS::WGM * TS::WGN);
    if (d.cut) {
        auto kern = k_gemm_dw<BITS, WT, AP, TS::BM, TS::BN, TS::BK, TS::NS, TS::WGM, TS::WGN, true>;
        static uint64_t attr_done = 0;
        allow_dynamic_lds(kern, smem, attr_done);
        kern<<<grid, block, smem, st>>>(a);
    } else {
        auto kern = k_gemm_dw<BITS, WT, AP, TS::BM, TS::BN, TS::BK, TS::NS, TS::WGM, TS::WGN, false>;
        static uint64_t attr_done = 0;
        allow_dynamic_lds(kern, smem, attr_done);
        kern<<<grid, block, smem, st>>>(a);
    }
}

template <typename WT, bool AP>
bool launch_dw_bits(int bits, const GemmDwArgs &a, const SkScratch &sk, hipStream_t st)   // returns whether per-segment partials were written
{
    const bool small = use_small_tile(a.I, a.O);
#define EQAT_GO(B) do { if (small) launch_dw_t<B, WT, AP, DwTileSmall>(a, sk, st); else launch_dw_t<B, WT, AP, DwTileBig>(a, sk, st); } while (0)
    if (bits == 2) EQAT_GO(2); else if (bits == 3) EQAT_GO(3); else EQAT_GO(4);
#undef EQAT_GO
    return ((small ? TileSmall::BM : TileBig::BM) % a.g) != 0;
}

}  // namespace

// workspace reservation: either tile shape may be picked at launch
bool dw_needs_partials(const Problem &p) { return (TileSmall::BM % p.g) != 0; }

// Scratch that cutting tiles along K needs, for whichever of the GEMMs of a problem may do so (bwd: fwd, dX and dW,
// else the forward alone): the largest of their needs, with the full complement of compute units.
void sk_scratch_bytes(const Problem &p, bool bwd, size_t *partial_bytes, size_t *counter_bytes)
{
    *partial_bytes = 0;
    *counter_bytes = p.act_bf16 ? (size_t)kSkCounterWords * sizeof(uint32_t) : 0;     // whatever the token count
    if (!p.act_bf16 || p.T == 0) return;
    float *const some_p = reinterpret_cast<float *>(16); uint32_t *const some_c = reinterpret_cast<uint32_t *>(16);
    auto one = [&](int64_t m, int64_t n, int64_t k, bool runs) {
        const bool small = use_small_tile(m, n);
        const int b = small ? TileSmall::BM : TileBig::BM, resident = kMaxCus * (small ? 2 : 1);
        const int ntiles = (int)(((m + b - 1) / b) * ((n + b - 1) / b));
        const SkPlan sk = plan_tiles(ntiles, (int)(((k + 63) / 64 + 1) / 2), resident, some_p, some_c, runs);
        if (!sk.walk) return;
        const int W = resident / 8, n_sk = (ntiles + 7) / 8 - sk.dp_rounds * W;
        if (n_sk <= 0) return;
        *partial_bytes = std::max(*partial_bytes, (size_t)resident * 2 * b * b * sizeof(float));
    };
    one(p.T, p.O, p.I, true);
    if (bwd) { one(p.T, p.I, p.O, true); one(p.I, p.O, p.T, false); }
}

// Test aid: work item number j of workgroup `block` in the launch that the forward (gemm = 0), the dX (gemm = 1) or the dW
// (gemm = 2; tile rows: in-features, tile columns: out-features, K: tokens) GEMM of this problem makes, as the kernel
// itself works it out.  item = {tile row, tile column, first and past-the-last K-tile pair, contributors of the tile, the
// first contributor's index in its XCD, 1 for a split tile, counter index, grid, K-tile pairs per tile, tile rows, tile
// columns}.  Returns 1, 0 past the workgroup's last item, -1 for a bad argument.
int plan_item_for_test(const Problem &p, int gemm, int block, int j, int32_t item[12])
{
    if (!p.act_bf16 || p.T < 1 || gemm < 0 || gemm > 2 || block < 0 || j < 0) return -1;
    if (gemm == 2) {
        float *const some_p = reinterpret_cast<float *>(16); uint32_t *const some_c = reinterpret_cast<uint32_t *>(16);
        const bool small = use_small_tile(p.I, p.O);
        const DwLaunchPlan d = small ? plan_dw<bf16_t, true, DwTileSmall>((int)p.I, (int)p.O, (int)p.T, some_p, some_c)
                                     : plan_dw<bf16_t, true, DwTileBig>((int)p.I, (int)p.O, (int)p.T, some_p, some_c);
        if (block >= d.grid) return -1;
        SkItem it{};
        bool ok;
        if (d.cut) {
            ok = sk_item_of(d.sk, d.ntiles, d.tiles_m, d.tiles_n, 8, block, d.grid, j, it);
        } else {        // one workgroup per tile
            ok = j == 0 && tile_of_xcd_slot(d.grid, block & 7, block >> 3, d.tiles_m, d.tiles_n, it.tm, it.tn, 8);
            it.kb = 0; it.ke = (((int)p.T + 63) / 64 + 1) / 2; it.parts = 1;
        }
        const int32_t v[12] = {it.tm, it.tn, it.kb, it.ke, it.parts, it.first, it.fixed, it.ctr, d.grid, (((int)p.T + 63) / 64 + 1) / 2, d.tiles_m, d.tiles_n};
        for (int k = 0; k < 12; ++k) item[k] = v[k];
        return ok ? 1 : 0;
    }
    const int M = (int)p.T, N = (int)(gemm == 0 ? p.O : p.I), K = (int)(gemm == 0 ? p.I : p.O);
    float *const some_p = reinterpret_cast<float *>(16); uint32_t *const some_c = reinterpret_cast<uint32_t *>(16);
    const bool small = use_small_tile(M, N);
    const QLaunchPlan q = gemm == 0 ? (small ? plan_q<false, TileSmall>(M, N, K, some_p, some_c) : plan_q<false, TileBig>(M, N, K, some_p, some_c))
                                    : (small ? plan_q<true, TileSmall>(M, N, K, some_p, some_c) : plan_q<true, TileBig>(M, N, K, some_p, some_c));
    if (block >= q.grid) return -1;
    SkItem it{};
    bool ok;
    if (q.cut_inst) {
        ok = sk_item_of(q.sk, q.ntiles, q.tiles_m, q.tiles_n, q.band, block, q.grid, j, it);
    } else {        // whole tiles only, as in the kernel's other instantiation
        const int loc_step = q.sk.walk ? q.grid >> 3 : q.ntiles;
        ok = tile_of_xcd_slot(q.sk.walk ? q.ntiles : q.grid, block & 7, (block >> 3) + j * loc_step, q.tiles_m, q.tiles_n, it.tm, it.tn, q.band);
        it.kb = 0; it.ke = q.sk.pairs; it.parts = 1;
    }
    const int32_t v[12] = {it.tm, it.tn, it.kb, it.ke, it.parts, it.first, it.fixed, it.ctr, q.grid, q.sk.pairs, q.tiles_m, q.tiles_n};
    for (int k = 0; k < 12; ++k) item[k] = v[k];
    return ok ? 1 : 0;
}

void launch_mfma_fwd(const Problem &p, const void *X, const void *codes, const void *sz, void *Y, const SkScratch &sk,
                     hipStream_t st)
{
    if (p.T == 0) return;
    GemmQArgs a{};
    a.sk.partials = sk.partials; a.sk.counters = sk.counters;
    a.A = (const bf16_t *)X; a.codes = (const uint32_t *)codes; a.sz = (const floatx2 *)sz; a.C = (bf16_t *)Y;
    a.M = (int)p.T; a.N = (int)p.O; a.K = (int)p.I; a.I = (int)p.I; a.G = (int)p.G; a.g = (int)p.g;
    a.a_bytes = (uint32_t)(p.T * p.I * 2); a.codes_bytes = (uint32_t)work_code_bytes(p); a.sz_bytes = (uint32_t)(p.O * p.G * 8);
    launch_q_bits<false>(p.bits, a, st);
}

void launch_mfma_dx(const Problem &p, const void *dY, const void *codes, const void *sz, void *dX, const SkScratch &sk,
                    hipStream_t st)
{
    if (p.T == 0) return;
    GemmQArgs a{};
    a.sk.partials = sk.partials; a.sk.counters = sk.counters;
    a.A = (const bf16_t *)dY; a.codes = (const uint32_t *)codes; a.sz = (const floatx2 *)sz; a.C = (bf16_t *)dX;
    a.M = (int)p.T; a.N = (int)p.I; a.K = (int)p.O; a.I = (int)p.I; a.G = (int)p.G; a.g = (int)p.g;
    a.a_bytes = (uint32_t)(p.T * p.O * 2); a.codes_bytes = (uint32_t)work_code_bytes(p); a.sz_bytes = (uint32_t)(p.O * p.G * 8);
    launch_q_bits<true>(p.bits, a, st);
}

void launch_mfma_dw(const Problem &p, bool block_ap, const void *X, const void *dY, const void *W, const void *codes,
                    const void *clampbits, const void *sz, const float *s, void *dW, float *ds, float *dz, float *part,
                    const SkScratch &sk, hipStream_t st)
{
    GemmDwArgs a{};
    a.X = (const bf16_t *)X; a.dY = (const bf16_t *)dY; a.W = W; a.codes = (const uint32_t *)codes;
    a.clampbits = (const uint8_t *)clampbits; a.sz = (const floatx2 *)sz;
    a.dW = dW; a.ds = ds; a.dz = dz;
    a.T = (int)p.T; a.I = (int)p.I; a.O = (int)p.O; a.G = (int)p.G; a.g = (int)p.g;
    a.x_bytes = (uint32_t)(p.T * p.I * 2); a.dy_bytes = (uint32_t)(p.T * p.O * 2);
    a.w_bytes = (uint32_t)(p.O * p.I * (p.w_bf16 ? 2 : 4)); a.codes_bytes = (uint32_t)work_code_bytes(p);
    a.clamp_bytes = (uint32_t)(p.O * p.I / 8); a.sz_bytes = (uint32_t)(p.O * p.G * 8);
    bool partials;
    const size_t n32 = (size_t)p.O * (p.I / 32);
    a.part_ds = part; a.part_dz = part ? part + n32 : nullptr;
    {
        ProfScope ps(PK_GEMM_DW, st);
        if (block_ap) {
            if (p.w_bf16) partials = launch_dw_bits<bf16_t, true>(p.bits, a, sk, st);
            else partials = launch_dw_bits<float, true>(p.bits, a, sk, st);
        } else {
            partials = launch_dw_bits<bf16_t, false>(p.bits, a, sk, st);
        }
    }
    if (partials) {
        ProfScope ps(PK_REDUCE, st);
        const uint32_t n_per = (uint32_t)(p.g / 32);
        if (ds != nullptr) launch_reduce_partials(a.part_ds, ds, s, (size_t)p.O * p.G, n_per, false, st);
        if (dz != nullptr) launch_reduce_partials(a.part_dz, dz, s, (size_t)p.O * p.G, n_per, true, st);
    }
}

}  // namespace eqat
