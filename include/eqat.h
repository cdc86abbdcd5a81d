/*
 * eqat.h  --  C ABI of the MI355X (gfx950) quantized-linear library for
 * EfficientQAT (arXiv 2407.11062).
 *
 * The library implements the layer both training phases of the paper run on
 * every step:
 *   Block-AP (Sec. 3.2):  W_int = clamp(round(W/s) + z, 0, 2^N - 1)   Eq.(1)
 *                         What  = (W_int - z) * s                     Eq.(2)
 *                         Y = X * What^T, and the backward of App. B.
 *   E2E-QP  (Sec. 3.3):   W_int frozen and packed at N bits; only Eq.(2) runs.
 *
 * Conventions (all entry points)
 *   Layout     Row-major, contiguous.  X [T,I], W [O,I] (row = output channel),
 *              s,z [O,G] with G = I/g, Y,dY [T,O], dX [T,I], dW [O,I],
 *              ds,dz [O,G].  Group j of row o covers columns [j*g,(j+1)*g).
 *   Memory     Every pointer is a DEVICE pointer owned by the caller, 16-byte
 *              aligned.  The library never allocates or frees device memory and
 *              keeps no pointer of the caller (the optional timing aid at the end
 *              of this header creates HIP event objects while it is switched on).
 *              Each tensor must be smaller than 2 GiB.
 *   Dtypes     X,Y,dY,dX have desc.act_dtype; W,dW have desc.w_dtype; s,z,ds,dz
 *              are always fp32.  act bf16 selects the MFMA path (needs O % 8 == 0);
 *              act fp32 selects the fp32 path.
 *   Shapes     I % 32 == 0; g > 0, g % 32 == 0, g | I (group = -1 means g = I);
 *              bits in {2,3,4}; T >= 0, O >= 1; with bf16 activations I, O < 2^22.
 *   Stream     `stream` is a hipStream_t (NULL = default stream).  All work is
 *              enqueued there; no call synchronises.  Outputs are overwritten.
 *   Workspace  Caller-provided scratch of at least eqat_workspace_bytes(desc, op)
 *              bytes, 256-byte aligned; contents undefined afterwards.
 *   Errors     Arguments are checked on the host before anything is launched and
 *              the first violation is returned; nothing is thrown or aborted.
 *   Numerics   round() is round-half-to-even of the correctly rounded binary32
 *              quotient w/s (bf16 weights are widened first), so integer codes
 *              and packed bytes are identical on every implementation.
 *              zbar = clamp(round(z), 0, 2^N-1) is used in place of z in every
 *              entry point (the zero point is stored at N bits when Block-AP ends,
 *              so the packed layer is exactly the layer Block-AP trained); the
 *              gradient passes straight through the rounding and the clamp.
 *              Preconditions (not checked): s a normal,
 *              finite, positive binary32 number (>= 2^-126; the min/max rule
 *              never gives less than 1e-10), |z| <= 2^20, all inputs finite.
 *   Determinism  Same inputs give bitwise the same outputs.
 */
#ifndef EQAT_H_
#define EQAT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EQAT_OK = 0,
    EQAT_ERR_NULL = 1,      /* a required pointer is NULL                        */
    EQAT_ERR_SHAPE = 2,     /* T < 0, I or O < 1, I % 32, O % 8 (bf16), >= 2 GiB */
                            /* or, with bf16 activations, I or O >= 2^22         */
    EQAT_ERR_BITS = 3,      /* bits not in {2,3,4}                               */
    EQAT_ERR_GROUP = 4,     /* group not -1 and (<= 0, % 32 != 0 or not | I)     */
    EQAT_ERR_DTYPE = 5,     /* unknown dtype value                               */
    EQAT_ERR_ALIGN = 6,     /* pointer not 16-byte (workspace: 256-byte) aligned */
    EQAT_ERR_WORKSPACE = 7, /* workspace missing or too small                    */
    EQAT_ERR_DEVICE = 8,    /* the HIP runtime refused a launch                  */
    EQAT_ERR_HYPER = 9      /* optimizer constants out of range                  */
} eqat_status;

typedef enum { EQAT_F32 = 0, EQAT_BF16 = 1 } eqat_dtype;

typedef enum {
    EQAT_OP_FQ_FWD = 0, EQAT_OP_FQ_BWD = 1, EQAT_OP_Q_FWD = 2, EQAT_OP_Q_BWD = 3,
    EQAT_OP_QP_FWD = 4, EQAT_OP_QP_BWD = 5      /* eqat_qlinear_fwd_prepared / _bwd_prepared */
} eqat_op;

/* What eqat_unpack_state reads: the workspace left by eqat_fq_linear_fwd_keep, the one left by
 * eqat_qlinear_fwd_keep, or a layer prepared by eqat_qlinear_prepare. */
typedef enum { EQAT_STATE_FQ_KEPT = 0, EQAT_STATE_Q_KEPT = 1, EQAT_STATE_PREPARED = 2 } eqat_state_kind;

typedef struct eqat_desc {
    int64_t tokens;        /* T                                                  */
    int64_t in_features;   /* I                                                  */
    int64_t out_features;  /* O                                                  */
    int32_t bits;          /* N                                                  */
    int32_t group;         /* g, or -1 for one group per row (per-channel)       */
    int32_t act_dtype;     /* eqat_dtype of X, Y, dY, dX                         */
    int32_t w_dtype;       /* eqat_dtype of W, dW                                */
} eqat_desc;

/* Host-only helpers.  Sizes are 0 for an invalid descriptor. */
const char *eqat_status_string(int status);
eqat_status eqat_validate_desc(const eqat_desc *d);
size_t eqat_packed_w_bytes(const eqat_desc *d);   /* O * I*N/8                     */
size_t eqat_packed_z_bytes(const eqat_desc *d);   /* O * 4*ceil(G*N/32)            */
size_t eqat_workspace_bytes(const eqat_desc *d, int op);

/*
 * Per-group initialisation of step sizes and zero points.  The paper does not
 * say how s and z start; this is the usual asymmetric min/max rule in binary32:
 *   s = max((max - min) / (2^N - 1), 1e-10),  z = clamp(round(-min / s), 0, 2^N - 1).
 * In: W [O,I].  Out: s, z [O,G].  d->tokens is ignored.
 */
eqat_status eqat_init_minmax(const eqat_desc *d, const void *W, float *s, float *z, void *stream);

/*
 * Block-AP forward (Sec. 3.2, Eqs.(1),(2)):  Y = X * What^T.
 * What is rebuilt from W, s, z on the fly and never stored.
 */
eqat_status eqat_fq_linear_fwd(const eqat_desc *d, const void *X, const void *W, const float *s,
                               const float *z, void *Y, void *ws, size_t ws_bytes, void *stream);

/*
 * Block-AP backward (App. B, Eqs.(3)-(5), straight-through estimator):
 *   dX = dY * What
 *   dW = (dY^T X) where 0 <= round(w/s)+zbar <= 2^N-1, else 0            Eq.(5)
 *   ds[o,j] = sum over group of (dY^T X) * { round(w/s) - w/s | -zbar | 2^N-1-zbar }   Eq.(3)
 *   dz[o,j] = sum over group of (dY^T X) * { 0 in range | -s outside }                 Eq.(4)
 * Eq.(4) is printed with -1; -s is the derivative of Eq.(2) for a zero point in
 * integer units, and the printed form equals dz / s.  The appendix writes the
 * upper bound as 2^(N-1); Eq.(1)'s 2^N - 1 is used.
 * Any of dX, dW, ds, dz may be NULL and is then skipped.
 */
eqat_status eqat_fq_linear_bwd(const eqat_desc *d, const void *X, const void *W, const float *s,
                               const float *z, const void *dY, void *dX, void *dW, float *ds, float *dz,
                               void *ws, size_t ws_bytes, void *stream);

/*
 * The same pair for a training step that runs both on unchanged (W, s, z): the forward leaves what Eq.(1) produced
 * (codes, which weights were clamped, the (s, zbar) pairs) in the workspace and the backward uses it instead of
 * running Eq.(1) a second time.  Both take a workspace of EQAT_OP_FQ_BWD size.  Precondition of _bwd_kept (not
 * checked): `ws` is untouched since eqat_fq_linear_fwd_keep ran on the same descriptor (any token count), W, s and z.
 * Results are bitwise those of eqat_fq_linear_fwd / eqat_fq_linear_bwd.  (With fp32 activations nothing is kept and
 * the backward works from W as always.)
 */
eqat_status eqat_fq_linear_fwd_keep(const eqat_desc *d, const void *X, const void *W, const float *s,
                                    const float *z, void *Y, void *ws, size_t ws_bytes, void *stream);
eqat_status eqat_fq_linear_bwd_kept(const eqat_desc *d, const void *X, const void *W, const float *s,
                                    const float *z, const void *dY, void *dX, void *dW, float *ds, float *dz,
                                    void *ws, size_t ws_bytes, void *stream);

/*
 * The forward of the pair above from kept state: `ws` holds what eqat_fq_linear_fwd_keep or eqat_fq_quantize_batched
 * left for the same descriptor, W, s and z (not checked), and Eq.(1) is not run again.  Bitwise eqat_fq_linear_fwd.
 */
eqat_status eqat_fq_linear_fwd_kept(const eqat_desc *d, const void *X, const void *W, const float *s,
                                    const float *z, void *Y, void *ws, size_t ws_bytes, void *stream);

/*
 * Several matrices in ONE launch.  The linears of a decoder block are a few tens of megabytes each; the memory-bound
 * passes over them (min/max, Eq.(1), packing) last 10-25 microseconds apiece when launched one by one, a good part of it
 * filling and draining the chip.  n: 1 .. EQAT_MAX_BATCH; descs: n descriptors (host); every other argument: a HOST
 * array of n device pointers (or sizes), entry i belonging to descs[i].  All descriptors must agree in bits
 * (EQAT_ERR_BITS) and in the dtypes (EQAT_ERR_DTYPE); shapes and group sizes may differ.  Results are bitwise those of
 * n single calls.
 *   eqat_init_minmax_batched   as eqat_init_minmax.
 *   eqat_pack_batched          as eqat_pack.
 *   eqat_fq_quantize_batched   Eq.(1) of n linears before their Block-AP forward and backward: leaves every ws[i]
 *                              (EQAT_OP_FQ_BWD size for descs[i], tokens included) as eqat_fq_linear_fwd_keep would, for
 *                              eqat_fq_linear_fwd_kept / eqat_fq_linear_bwd_kept.  With fp32 activations nothing is kept
 *                              and nothing is launched.
 */
#define EQAT_MAX_BATCH 8
eqat_status eqat_init_minmax_batched(int n, const eqat_desc *descs, const void *const *W, float *const *s,
                                     float *const *z, void *stream);
eqat_status eqat_pack_batched(int n, const eqat_desc *descs, const void *const *W, const float *const *s,
                              const float *const *z, uint8_t *const *Wpacked, uint8_t *const *zpacked, void *stream);
eqat_status eqat_fq_quantize_batched(int n, const eqat_desc *descs, const void *const *W, const float *const *s,
                                     const float *const *z, void *const *ws, const size_t *ws_bytes, void *stream);

/*
 * Freeze after Block-AP (Sec. 3.2 last paragraph; App. E): W_q and z at N bits.
 * Layout (the paper fixes none): each row is a little-endian bit stream, code i
 * of the row in bits [i*N,(i+1)*N), stored as bytes, least significant first.
 *   Wpacked [O, I*N/8] bytes, zpacked [O, 4*ceil(G*N/32)] bytes (tail bits 0).
 * zbar = clamp(round(z), 0, 2^N-1) as in the Block-AP calls.  d->tokens is ignored.
 */
eqat_status eqat_pack(const eqat_desc *d, const void *W, const float *s, const float *z,
                      uint8_t *Wpacked, uint8_t *zpacked, void *stream);

/* Test aid: expand the packed streams to int32 codes [O,I] and zero points [O,G]
 * (either output may be NULL). */
eqat_status eqat_unpack(const eqat_desc *d, const uint8_t *Wpacked, const uint8_t *zpacked,
                        int32_t *codes, int32_t *zcodes, void *stream);

/*
 * E2E-QP forward (Sec. 3.3): What = (w_q - z) * s from the packed codes, Y = X * What^T.
 * With bf16 activations and at most 16 tokens (T * I * 2 <= 64 KiB) this is one memory-bound
 * matrix-vector kernel that reads the packed arrays as they are and uses no workspace (the
 * decode-time case of the paper's App. "Speedup with BitBLAS"); otherwise the tiled MFMA GEMM.
 */
eqat_status eqat_qlinear_fwd(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                             const uint8_t *zpacked, void *Y, void *ws, size_t ws_bytes, void *stream);

/*
 * E2E-QP backward (Sec. 3.3): dX = dY * What and
 *   ds[o,j] = sum over group of (dY^T X)[o,i] * (w_q[o,i] - z[o,j]).
 * dX or ds may be NULL (skipped).  d->w_dtype is ignored.
 */
eqat_status eqat_qlinear_bwd(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                             const uint8_t *zpacked, const void *dY, void *dX, float *ds,
                             void *ws, size_t ws_bytes, void *stream);

/*
 * The E2E-QP pair for a training step that runs forward and backward on unchanged (Wpacked, s, zpacked): the forward
 * leaves the codes in the library's working layout and the (s, z) pairs in the workspace, the backward uses them.
 * Both take a workspace of EQAT_OP_Q_BWD size; the forward always runs the tiled GEMM (no few-token kernel).
 * Precondition of _bwd_kept (not checked): `ws` untouched since eqat_qlinear_fwd_keep ran on the same descriptor (any
 * token count), Wpacked, s and zpacked.  Results are bitwise those of eqat_qlinear_fwd (more than 16 tokens) /
 * eqat_qlinear_bwd.
 */
eqat_status eqat_qlinear_fwd_keep(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                                  const uint8_t *zpacked, void *Y, void *ws, size_t ws_bytes, void *stream);
eqat_status eqat_qlinear_bwd_kept(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                                  const uint8_t *zpacked, const void *dY, void *dX, float *ds,
                                  void *ws, size_t ws_bytes, void *stream);

/*
 * E2E-QP on a layer prepared once (Sec. 3.3: W_q is frozen in this phase and only s, or s and z, train).  The codes are
 * brought into the layout the GEMM kernels read and the packed zero points become floats, one time; a call then runs its
 * GEMMs behind one small launch that pairs the current step sizes with the zero points (O*G pairs: s changes every step).
 *   eqat_prepared_bytes    size of the prepared layer for this descriptor (tokens ignored; act_dtype matters:
 *                          with fp32 activations the prepared layer holds the dense stream); 0 for a bad descriptor.
 *   eqat_qlinear_prepare   Wpacked, zpacked (as eqat_pack wrote them) -> prepared (device, 256-byte aligned, owned by
 *                          the caller, at least eqat_prepared_bytes; too small gives EQAT_ERR_WORKSPACE).  Enqueues one
 *                          kernel (and, with fp32 activations, one device-to-device copy).
 *   eqat_qlinear_fwd_prepared / _bwd_prepared
 *                          Y, and dX / ds / dz, exactly (bitwise) as eqat_qlinear_fwd / eqat_qlinear_bwd, or, with a
 *                          float array z [O,G] given, as eqat_qlinear_fwd_z / eqat_qlinear_bwd_z.  z NULL: the zero
 *                          points the layer was prepared with.  dz = -s * group-sum (dY^T X) may be asked for either way.
 *                          Workspace of EQAT_OP_QP_FWD / EQAT_OP_QP_BWD size (the pairs; no room for codes).
 *                          The tiled GEMM always runs (no few-token kernel).  The prepared layer is only read, except for
 *                          a few counters inside it that a launch uses and leaves at zero: calls on the same prepared
 *                          layer must not overlap in time (different streams need their own copy).
 *   eqat_qlinear_fwd_prepared_keep / eqat_qlinear_bwd_prepared_kept
 *                          The same two calls for a training step that runs both on unchanged (s, z): the forward takes
 *                          a workspace of EQAT_OP_QP_BWD size and leaves the pairs in it; the backward, given the same
 *                          workspace untouched and the same s and z, skips the pairing launch.  Results are bitwise
 *                          those of the plain pair.  With tokens = 0 the _keep call still writes the pairs.
 */
size_t eqat_prepared_bytes(const eqat_desc *d);
eqat_status eqat_qlinear_prepare(const eqat_desc *d, const uint8_t *Wpacked, const uint8_t *zpacked, void *prepared,
                                 size_t prepared_bytes, void *stream);
eqat_status eqat_qlinear_fwd_prepared(const eqat_desc *d, const void *X, const void *prepared, const float *s,
                                      const float *z, void *Y, void *ws, size_t ws_bytes, void *stream);
eqat_status eqat_qlinear_bwd_prepared(const eqat_desc *d, const void *X, const void *prepared, const float *s,
                                      const float *z, const void *dY, void *dX, float *ds, float *dz,
                                      void *ws, size_t ws_bytes, void *stream);
eqat_status eqat_qlinear_fwd_prepared_keep(const eqat_desc *d, const void *X, const void *prepared, const float *s,
                                      const float *z, void *Y, void *ws, size_t ws_bytes, void *stream);
eqat_status eqat_qlinear_bwd_prepared_kept(const eqat_desc *d, const void *X, const void *prepared, const float *s,
                                      const float *z, const void *dY, void *dX, float *ds, float *dz,
                                      void *ws, size_t ws_bytes, void *stream);

/*
 * Test aid: the integer state the GEMM kernels work from, in plain arrays.  `kind` (eqat_state_kind) says what `state` is.
 *   codes   int32 [O,I]   W_int of Eq.(1) (Block-AP) or the frozen w_q (E2E-QP), or NULL
 *   clamped uint8 [O,I]   1 where Eq.(1) clamped the weight, i.e. where Eq.(5) zeroes dW; EQAT_STATE_FQ_KEPT only
 *                         (EQAT_ERR_NULL if asked of another kind), or NULL
 *   zbar    float [O,G]   the zero point Eq.(2) uses: clamp(round(z), 0, 2^N-1), or the unpacked N-bit zero point; or NULL
 * bf16 activations only (the fp32 path keeps no such state): EQAT_ERR_DTYPE otherwise.  d->tokens is ignored.
 */
eqat_status eqat_unpack_state(const eqat_desc *d, int kind, const void *state, int32_t *codes, uint8_t *clamped,
                              float *zbar, void *stream);

/*
 * E2E-QP with trained zero points (Sec. 3.3 and the ablation on the trainable parameters of E2E-QP: training z
 * promotes it from N bits to a floating-point tensor).  There is no Eq.(1) in this phase, so z enters Eq.(2) as it
 * is, WITHOUT rounding:  What = (w_q - z) * s,  Y = X * What^T.
 *   z [O,G] fp32 (device), any finite value.  Everything else as eqat_qlinear_fwd; workspace of EQAT_OP_Q_FWD.
 */
eqat_status eqat_qlinear_fwd_z(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                               const float *z, void *Y, void *ws, size_t ws_bytes, void *stream);

/*
 * Backward of the above:  dX = dY * What,
 *   ds[o,j] = sum over group of (dY^T X)[o,i] * (w_q[o,i] - z[o,j]),
 *   dz[o,j] = -s[o,j] * sum over group of (dY^T X)[o,i]            (derivative of Eq.(2) with respect to z).
 * dX, ds, dz may each be NULL (skipped).  Workspace of EQAT_OP_Q_BWD.  d->w_dtype is ignored.
 */
eqat_status eqat_qlinear_bwd_z(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                               const float *z, const void *dY, void *dX, float *ds, float *dz,
                               void *ws, size_t ws_bytes, void *stream);

/*
 * Block-AP step glue.  Sec. 3.2 trains the quantized block against the output of its full-precision counterpart with
 * a reconstruction loss; Sec. 4.1 ("Training") gives one learning rate for the quantization parameters and another
 * for the weights.  The paper names neither the form of the loss nor the optimizer; taken here: the mean squared
 * error over all elements, and AdamW (bias-corrected Adam with decoupled weight decay).
 *
 * eqat_recon_loss:   loss[0] = (1/n) sum (Y - Yref)^2,   dY = 2 (Y - Yref) / n   (dY may be NULL; it must not overlap Y or Yref).
 *   Y, Yref, dY: n elements of `dtype` (eqat_dtype), device, 16-byte aligned; loss: one float, device.
 *   ws: eqat_recon_loss_workspace_bytes() bytes, 256-byte aligned.  The sum is taken in a fixed order in binary32.
 *   n < 1 gives EQAT_ERR_SHAPE.
 */
size_t eqat_recon_loss_workspace_bytes(void);
eqat_status eqat_recon_loss(int64_t n, int32_t dtype, const void *Y, const void *Yref, float *loss, void *dY,
                            void *ws, size_t ws_bytes, void *stream);

/*
 * eqat_recon_loss for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving or training loops, harnesses that forbid hipMalloc.  Same kernels, same results (bitwise) as
 * eqat_recon_loss; the workgroup partials live in an 8 KiB array inside the library's device image (one copy per GPU,
 * held until the process ends) instead of `ws`.  The call allocates and frees nothing.
 *   Limit: none on n; the array holds the 2048 partials that are the most a launch ever uses (a library built with a
 *   larger eqat_recon_loss_workspace_bytes() returns EQAT_ERR_WORKSPACE here).
 *   The address of the array is looked up on the first call on each device (hipGetSymbolAddress; failure gives
 *   EQAT_ERR_DEVICE): make that first call outside stream capture.
 *   All calls on one GPU share the array: calls that may run at the same time on one GPU (different streams) race on
 *   it and must be ordered by the caller.  Nothing needs clearing between calls.
 */
eqat_status eqat_recon_loss_static(int64_t n, int32_t dtype, const void *Y, const void *Yref, float *loss, void *dY,
                                   void *stream);

/*
 * eqat_block_ap_update: one AdamW step, in place, on the three trained tensors of a linear in ONE launch, taking the
 * gradients as eqat_fq_linear_bwd wrote them (dW in W's dtype, ds and dz fp32).  Per element, in binary32:
 *   p <- p - lr wd p;  m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
 *   p <- p - lr (m / (1 - b1^step)) / (sqrt(v / (1 - b2^step)) + eps)          (then s <- max(s, 1e-10), see below)
 * with lr = lr_w, wd = weight_decay_w for W and lr_q, weight_decay_q for s and z.  Moments are fp32 arrays of the
 * parameter's shape, zero before the first step, owned by the caller.  A NULL parameter pointer (W, s or z) skips that
 * tensor together with its gradient and moments (E2E-QP trains s alone).  d->tokens and d->act_dtype are ignored.
 * A bf16 W is rounded to nearest even after the update; steps smaller than half an ulp are lost, so W should be kept
 * in fp32 while it is trained.  Constants outside 0 <= beta < 1, eps >= 0, step >= 1 give EQAT_ERR_HYPER.
 * The updated step sizes are held at or above 1e-10, the floor of their min/max initialisation (Eq.(1) divides by s, and
 * nothing else keeps an optimizer step from crossing zero): s <- max(s, 1e-10).
 */
typedef struct eqat_adamw {
    float lr_w;             /* learning rate of the weights (Sec. 4.1: 2e-5 at 2 bit, 1e-5 at 3 and 4 bit)   */
    float lr_q;             /* learning rate of step sizes and zero points (Sec. 4.1: 1e-4)                  */
    float beta1, beta2, eps;
    float weight_decay_w, weight_decay_q;
    int32_t step;           /* number of this update, counted from 1                                         */
} eqat_adamw;
eqat_status eqat_block_ap_update(const eqat_desc *d, const eqat_adamw *h, void *W, float *s, float *z,
                                 const void *dW, const float *ds, const float *dz, float *mW, float *vW,
                                 float *ms, float *vs, float *mz, float *vz, void *stream);

/*
 * Test aid (host only, nothing is launched): how the forward (gemm = 0), dX (gemm = 1) or dW (gemm = 2: tile rows are
 * in-features, tile columns out-features, K runs over the tokens) GEMM of this descriptor (bf16 activations, tokens >= 1)
 * divides its output tiles and their K range among its workgroups, as the kernel itself works it out.  item[12] = { tile row, tile column, first and past-the-last K-tile pair of this piece,
 * number of workgroups that contribute to the tile, index of the first of them within its XCD (workgroup = index * 8 +
 * XCD, XCD = block % 8), 1 if the tile is split among a group of workgroups (else pieces come from runs), index of the
 * tile's counter, workgroups in the launch, K-tile pairs per tile, tile rows, tile columns }; *exists = 0 past the last
 * item j of workgroup `block`.  EQAT_ERR_SHAPE for block outside the launch, gemm not 0, 1 or 2, j < 0.  Lets a test check,
 * without a GPU, that every K-tile pair of every tile is computed exactly once for any shape.
 */
eqat_status eqat_plan_item(const eqat_desc *d, int gemm, int block, int j, int32_t *item, int32_t *exists);

/*
 * Optional per-kernel timing (measurement aid, not part of the paper's method).
 * Between eqat_profile_start() and eqat_profile_stop() every kernel launch of the
 * library is bracketed by a pair of HIP events recorded on the caller's stream.
 * eqat_profile_stop() waits for those events and writes, per kernel class k in
 * [0, eqat_profile_kernels()), the summed elapsed milliseconds and the number of
 * launches into host arrays of length n; it then switches timing off.  Event
 * objects are created on first use and kept until the process ends.  The calls
 * may come from several threads; a session is process-wide (one start, one stop).
 */
int eqat_profile_kernels(void);
const char *eqat_profile_kernel_name(int k);
eqat_status eqat_profile_start(void);
eqat_status eqat_profile_stop(double *total_ms, int64_t *launches, int n);

#ifdef __cplusplus
}
#endif
#endif /* EQAT_H_ */
