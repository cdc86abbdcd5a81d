// Internal launcher interface between the C ABI (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/eqat.h"

namespace eqat {

struct Problem {
    int64_t T, I, O, g, G;
    int bits;
    bool act_bf16, w_bf16;
};

// ---- quant.hip -------------------------------------------------------------------------------
// Eq.(1): W,s,z -> codes (+ optional clamp bit-plane [O,I/8] bytes, + optional (s,zbar) pairs [O,G]).
// for_pack: the dense stream of the C ABI; otherwise the working layout the GEMM kernels read (work_code_bytes()).
// zpacked (may be NULL): the zero points at N bits are packed by extra workgroups of the same launch.
// zero_words (may be NULL): n_zero 32-bit words that the launch also clears (the arrival counters of the GEMMs).
void launch_quantize(const Problem &p, const void *W, const float *s, const float *z, void *codes, void *clampbits,
                     void *sz, void *zpacked, bool for_pack, uint32_t *zero_words, uint32_t n_zero, hipStream_t st);
// The same for up to kMaxBatch matrices in ONE launch; all jobs share bits, the weight dtype, and whether a clamp plane
// is written (the first job decides).
constexpr int kMaxBatch = EQAT_MAX_BATCH;
struct QuantizeJob {
    Problem p; const void *W; const float *s, *z; void *codes, *clampbits, *sz, *zpacked; uint32_t *zero_words; uint32_t n_zero;
};
void launch_quantize_batch(const QuantizeJob *jobs, int n, bool for_pack, hipStream_t st);
struct InitJob { Problem p; const void *W; float *s, *z; };
void launch_init_minmax_batch(const InitJob *jobs, int n, hipStream_t st);       // all jobs share bits and the weight dtype
inline size_t work_code_bytes(const Problem &p) { return (size_t)p.O * p.I / (p.bits == 2 ? 4 : 2); }
// One launch before the GEMMs of an E2E-QP call: dense stream -> working layout (packed == NULL: skipped) and the
// (s, z) pairs (sz == NULL: skipped), z taken from the packed N-bit zero points or from a float array (exactly one of
// the two not NULL); zb_out (may be NULL) receives the zero points alone, as floats.
void launch_e2e_prepare(const Problem &p, const void *packed, void *work, const float *s, const void *zpacked,
                        const float *zfloat, void *sz, float *zb_out, uint32_t *zero_words, uint32_t n_zero, hipStream_t st);
// Test aid: working-layout codes -> int32 [O,I]; clamp bit-plane -> bytes 0/1 [O,I]; (s, zero point) pairs -> the
// zero points [O,G] (each output may be NULL).
void launch_unpack_work(const Problem &p, const void *work, const void *clampbits, const void *sz, int32_t *codes,
                        uint8_t *clamped, float *zbar, hipStream_t st);
void launch_unpack(const Problem &p, const void *Wpacked, const void *zpacked, int32_t *codes, int32_t *zcodes, hipStream_t st);
void launch_init_minmax(const Problem &p, const void *W, float *s, float *z, hipStream_t st);
void launch_reduce_partials(const float *part, float *out, const float *s, size_t n_out, uint32_t n_per, bool scale_by_s,
                            hipStream_t st);

// ---- gemm_mfma.hip (bf16 activations) -----------------------------------------------------------
// Scratch of the GEMM launches that cut the tiles of a partly filled last round along K: one buffer of fp32 accumulator
// tiles and one arrival counter per tile.  The counters must be zero when a launch starts; every launch leaves them zero.
// Either pointer NULL: tiles are never cut.
struct SkScratch { float *partials; uint32_t *counters; };
int plan_item_for_test(const Problem &p, int gemm, int block, int j, int32_t item[12]);      // test aid, see gemm_mfma.hip
void sk_scratch_bytes(const Problem &p, bool bwd, size_t *partial_bytes, size_t *counter_bytes);
// Y[T,O] = X[T,I] * What[O,I]^T with What = (code - zbar) * s rebuilt per tile from packed codes.
void launch_mfma_fwd(const Problem &p, const void *X, const void *codes, const void *sz, void *Y, const SkScratch &sk,
                     hipStream_t st);
// dX[T,I] = dY[T,O] * What[O,I]
void launch_mfma_dx(const Problem &p, const void *dY, const void *codes, const void *sz, void *dX, const SkScratch &sk,
                    hipStream_t st);
// dWhat = dY^T X fused with the per-element / per-group epilogue.
//   block_ap: needs W, clampbits; writes dW (W's dtype, may be NULL), ds, dz (may be NULL).
//   e2e_qp  : W = clampbits = dW = NULL; writes ds and, if not NULL, dz = -s * group-sum dWhat.
// `part` is scratch for [2][O, I/32] floats, used only when a group is wider than one tile (see dw_needs_partials);
// `sk` is the scratch of launches that cut tiles along T.
void launch_mfma_dw(const Problem &p, bool block_ap, const void *X, const void *dY, const void *W, const void *codes,
                    const void *clampbits, const void *sz, const float *s, void *dW, float *ds, float *dz, float *part,
                    const SkScratch &sk, hipStream_t st);
bool dw_needs_partials(const Problem &p);

// ---- gemv.hip (E2E-QP forward for a few tokens, straight from the dense packed stream) -----------
bool gemv_applies(const Problem &p);
// exactly one of zpacked / zfloat is not NULL
void launch_gemv(const Problem &p, const void *X, const void *Wpacked, const float *s, const void *zpacked,
                 const float *zfloat, void *Y, hipStream_t st);

// ---- train_step.hip (Block-AP step glue: reconstruction loss, AdamW over {W, s, z}) --------------------
size_t recon_loss_ws_bytes();
// loss[0] = mean (Y - Yref)^2, dY (may be NULL) = 2 (Y - Yref) / n; `partial` = recon_loss_ws_bytes() of scratch.
void launch_recon_loss(int64_t n, bool bf16, const void *Y, const void *Yref, float *loss, void *dY, float *partial,
                       hipStream_t st);
struct AdamGroup {                      // one parameter tensor; p == NULL: absent
    void *p; const void *g; float *m; float *v;
    int64_t n;
    float lr, weight_decay;
    bool bf16;                          // dtype of p and g (moments are always fp32)
    float p_min;                        // lower bound of the updated parameter (-inf: none)
};
// One launch over three parameter groups (weights, step sizes, zero points); step counts from 1.
void launch_adamw(const AdamGroup *groups, float beta1, float beta2, float eps, int step, hipStream_t st);

// ---- gemm_f32.hip (fp32 activations; simple tiled FMA kernels, exact division everywhere) --------
void launch_f32_fwd(const Problem &p, bool packed, const void *X, const void *W_or_codes, const float *s, const void *z_or_sz,
                    void *Y, hipStream_t st);
void launch_f32_dx(const Problem &p, bool packed, const void *dY, const void *W_or_codes, const float *s, const void *z_or_sz,
                   void *dX, hipStream_t st);
// dWhat[O,I] fp32 = dY^T X into `dwhat` (scratch O*I floats), then the per-group epilogue.
void launch_f32_dw(const Problem &p, bool block_ap, const void *X, const void *dY, const void *W_or_codes, const float *s,
                   const void *z_or_sz, float *dwhat, void *dW, float *ds, float *dz, hipStream_t st);

}  // namespace eqat
