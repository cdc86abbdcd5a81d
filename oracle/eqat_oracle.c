/*
 * EfficientQAT quantized-linear ORACLE  --  test infrastructure, not product.
 *
 * A plain, slow, single-file CPU implementation of what the quantized linear
 * layer of EfficientQAT (arXiv 2407.11062) computes, written directly from
 * the paper's equations.  It exists only so that the HIP library can be
 * checked against something that can be read next to the paper by eye.
 * Only tests, the smoke check and the benchmark's "cpu_baseline" leg may call
 * it; the product path never does.  It shares no code with the GPU library.
 *
 * Arithmetic: every sum and product is fp64.  The ONE exception is the
 * quantisation decision: Eq.(1) needs round(w/s), and an integer code must be
 * identical on every implementation, so the quotient is defined as the IEEE
 * binary32 correctly-rounded quotient of the binary32 values w and s, rounded
 * to the nearest integer with ties to even.  Inputs arrive as binary32 arrays
 * (bf16 data is widened exactly by the caller).
 *
 * Notation follows the paper: W [O x I] full-precision weights (row = output
 * channel), s and z [O x G] step size and zero point of each group of g
 * consecutive weights along the input dimension (G = I/g), N bits,
 * Qmax = 2^N - 1, X [T x I] activations, Y [T x O] = X * What^T.
 *
 * Readings of the paper taken here (each is listed in the design notes):
 *  - Appendix B writes the upper clamp bound as 2^{N-1}; Eq.(1) clamps to
 *    2^N - 1.  Differentiating Eq.(2) o Eq.(1) gives the appendix formulas
 *    with 2^N - 1, so Qmax = 2^N - 1 is used everywhere.
 *  - Eq.(4) prints d what / d z = -1 outside the clamp range.  The derivative
 *    of Eq.(2) with W_int pinned at a clamp bound is -s (z is in integer
 *    units); -s is used.  The printed form is dz / s.
 *  - z is learnable, yet W_int must be an integer and z is stored at N bits
 *    once Block-AP ends (Sec. 3.2 last paragraph; the N/g term of App. E's
 *    bits per parameter), and E2E-QP starts from exactly the model Block-AP
 *    trained (Sec. 3.3).  So the zero point Eqs.(1),(2) use must be one that
 *    N bits can hold: zbar = clamp(round_half_even(z), 0, Qmax) everywhere,
 *    in the fake-quant forward and backward as well as in the packed file,
 *    with the gradient passed straight through both the rounding and the
 *    clamp (d zbar / d z = 1).
 *  - The in-range condition is taken on round(w/s) + zbar BEFORE clamping,
 *    bounds inclusive, exactly as the case conditions of Eqs.(3)-(5) read.
 *
 * All functions return 0 on success, a negative number on a bad argument.
 * Parallelism: an OpenMP "parallel for" over independent output rows only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef long long i64;

int eqo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int bad_shape(i64 I, i64 O, int bits, i64 g)
{
    if (I <= 0 || O <= 0) return 1;
    if (bits < 1 || bits > 8) return 1;
    if (g <= 0 || I % g != 0) return 1;
    return 0;
}

/* ---- Eq.(1): one weight -> pre-clamp integer, code, fp32 quotient ------- */

typedef struct {
    float t;      /* binary32 quotient w/s                                   */
    double r;     /* round_half_even(t)                                      */
    double qpre;  /* r + zbar, before the clamp                              */
    double q;     /* clamp(qpre, 0, Qmax): the integer code W_int            */
    int side;     /* -1: qpre < 0, 0: in range, +1: qpre > Qmax              */
} quant1;

static quant1 quantize_one(float w, float s, double zbar, double qmax)
{
    quant1 a;
    a.t = w / s;                 /* binary32 division, correctly rounded     */
    a.r = rint((double)a.t);     /* ties to even (default rounding mode)     */
    a.qpre = a.r + zbar;
    a.side = 0;
    a.q = a.qpre;
    if (a.qpre < 0.0)  { a.side = -1; a.q = 0.0; }
    if (a.qpre > qmax) { a.side = +1; a.q = qmax; }
    return a;
}

static double zbar_of(float z, double qmax)
{
    double zb = rint((double)z);
    if (zb < 0.0) zb = 0.0;
    if (zb > qmax) zb = qmax;
    return zb;
}

/* ---- per-group min/max initialisation of s and z ------------------------- */
/* Not in the paper (it never says how s, z start); the usual asymmetric
 * min/max rule, all in binary32 so that s and z are reproducible bit for bit:
 *   s = max((wmax - wmin) / Qmax, 1e-10),  z = clamp(round(-wmin / s), 0, Qmax) */
int eqo_init_minmax(const float *W, i64 O, i64 I, int bits, i64 g, float *s, float *z)
{
    if (!W || !s || !z || bad_shape(I, O, bits, g)) return -1;
    const i64 G = I / g;
    const float qmax = (float)((1 << bits) - 1);
#pragma omp parallel for schedule(static)
    for (i64 o = 0; o < O; ++o) {
        for (i64 j = 0; j < G; ++j) {
            const float *w = W + o * I + j * g;
            float lo = w[0], hi = w[0];
            for (i64 k = 1; k < g; ++k) {
                if (w[k] < lo) lo = w[k];
                if (w[k] > hi) hi = w[k];
            }
            float range = hi - lo;
            float step = range / qmax;
            if (!(step >= 1e-10f)) step = 1e-10f;
            float zf = rintf((-lo) / step);
            if (zf < 0.0f) zf = 0.0f;
            if (zf > qmax) zf = qmax;
            s[o * G + j] = step;
            z[o * G + j] = zf;
        }
    }
    return 0;
}

/* ---- Eq.(1) over a matrix: codes and clamp side --------------------------- */
/* codes[o,i] = W_int in [0, Qmax]; side[o,i] in {-1,0,+1} (may be NULL).     */
int eqo_quantize(const float *W, const float *s, const float *z, i64 O, i64 I, int bits, i64 g,
                 int32_t *codes, int8_t *side)
{
    if (!W || !s || !z || !codes || bad_shape(I, O, bits, g)) return -1;
    const i64 G = I / g;
    const double qmax = (double)((1 << bits) - 1);
#pragma omp parallel for schedule(static)
    for (i64 o = 0; o < O; ++o)
        for (i64 i = 0; i < I; ++i) {
            const i64 j = i / g;
            quant1 a = quantize_one(W[o * I + i], s[o * G + j], zbar_of(z[o * G + j], qmax), qmax);
            codes[o * I + i] = (int32_t)a.q;
            if (side) side[o * I + i] = (int8_t)a.side;
        }
    return 0;
}

/* ---- Eq.(2) o Eq.(1): What = (W_int - zbar) * s --------------------------- */
static void dequant_row(const float *Wrow, const float *srow, const float *zrow, i64 I, i64 g,
                        double qmax, double *out)
{
    for (i64 i = 0; i < I; ++i) {
        const i64 j = i / g;
        const double zb = zbar_of(zrow[j], qmax);
        quant1 a = quantize_one(Wrow[i], srow[j], zb, qmax);
        out[i] = (a.q - zb) * (double)srow[j];
    }
}

int eqo_fake_quant(const float *W, const float *s, const float *z, i64 O, i64 I, int bits, i64 g,
                   double *What)
{
    if (!W || !s || !z || !What || bad_shape(I, O, bits, g)) return -1;
    const i64 G = I / g;
    const double qmax = (double)((1 << bits) - 1);
#pragma omp parallel for schedule(static)
    for (i64 o = 0; o < O; ++o)
        dequant_row(W + o * I, s + o * G, z + o * G, I, g, qmax, What + o * I);
    return 0;
}

/* ---- Block-AP forward: Y = X * What^T (Sec. 3.2, Eqs.(1),(2)) ------------- */
int eqo_fq_linear_fwd(const float *X, const float *W, const float *s, const float *z,
                      i64 T, i64 I, i64 O, int bits, i64 g, double *Y)
{
    if (!W || !s || !z || bad_shape(I, O, bits, g) || T < 0) return -1;
    if (T == 0) return 0;
    if (!X || !Y) return -1;
    const i64 G = I / g;
    const double qmax = (double)((1 << bits) - 1);
    int fail = 0;
#pragma omp parallel
    {
        double *wh = (double *)malloc((size_t)I * sizeof(double));
        if (!wh) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (i64 o = 0; o < O; ++o) {
            if (!wh) continue;
            dequant_row(W + o * I, s + o * G, z + o * G, I, g, qmax, wh);
            for (i64 t = 0; t < T; ++t) {
                const float *x = X + t * I;
                double acc = 0.0;
                for (i64 i = 0; i < I; ++i) acc += (double)x[i] * wh[i];
                Y[t * O + o] = acc;
            }
        }
        free(wh);
    }
    return fail ? -2 : 0;
}

/* dX[t,i] = sum_o dY[t,o] * What[o,i], with What given as a dense fp64 matrix */
static void dx_from_what(const float *dY, const double *What, i64 T, i64 I, i64 O, double *dX)
{
#pragma omp parallel for schedule(static)
    for (i64 t = 0; t < T; ++t) {
        double *dx = dX + t * I;
        for (i64 i = 0; i < I; ++i) dx[i] = 0.0;
        for (i64 o = 0; o < O; ++o) {
            const double a = (double)dY[t * O + o];
            const double *wh = What + o * I;
            for (i64 i = 0; i < I; ++i) dx[i] += a * wh[i];
        }
    }
}

/* dWhat[o,:] = sum_t dY[t,o] * X[t,:] for one output row */
static void dwhat_row(const float *X, const float *dY, i64 T, i64 I, i64 O, i64 o, double *acc)
{
    for (i64 i = 0; i < I; ++i) acc[i] = 0.0;
    for (i64 t = 0; t < T; ++t) {
        const double a = (double)dY[t * O + o];
        const float *x = X + t * I;
        for (i64 i = 0; i < I; ++i) acc[i] += a * (double)x[i];
    }
}

/* ---- Block-AP backward (App. B, Eqs.(3)-(5), chain rule through Eq.(2)) ----
 *   dX = dY * What
 *   dWhat = dY^T * X
 *   dW[o,i] = dWhat[o,i] * (in range ? 1 : 0)                         Eq.(5)
 *   ds[o,j] = sum_{i in group j} dWhat[o,i] * cs,
 *        cs = round(w/s) - w/s   in range
 *             -zbar              below the range
 *             Qmax - zbar        above the range                      Eq.(3)
 *   dz[o,j] = sum_{i in group j} dWhat[o,i] * cz,  cz = 0 in range, -s outside
 *                                                                      Eq.(4)
 * Any of dX, dW, ds, dz may be NULL (skipped).  X may be NULL when only dX
 * is wanted.                                                                  */
int eqo_fq_linear_bwd(const float *X, const float *W, const float *s, const float *z,
                      const float *dY, i64 T, i64 I, i64 O, int bits, i64 g,
                      double *dX, double *dW, double *ds, double *dz)
{
    if (!W || !s || !z || bad_shape(I, O, bits, g) || T < 0) return -1;
    if (T > 0 && !dY) return -1;
    const i64 G = I / g;
    const double qmax = (double)((1 << bits) - 1);
    const int want_w = (dW || ds || dz);
    if (want_w && T > 0 && !X) return -1;

    if (dX && T > 0) {
        double *What = (double *)malloc((size_t)O * (size_t)I * sizeof(double));
        if (!What) return -2;
        eqo_fake_quant(W, s, z, O, I, bits, g, What);
        dx_from_what(dY, What, T, I, O, dX);
        free(What);
    }
    if (!want_w) return 0;

    int fail = 0;
#pragma omp parallel
    {
        double *acc = (double *)malloc((size_t)I * sizeof(double));
        if (!acc) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (i64 o = 0; o < O; ++o) {
            if (!acc) continue;
            dwhat_row(X, dY, T, I, O, o, acc);
            for (i64 j = 0; j < G; ++j) {
                const float sj = s[o * G + j];
                const double zb = zbar_of(z[o * G + j], qmax);
                double gs = 0.0, gz = 0.0;
                for (i64 i = j * g; i < (j + 1) * g; ++i) {
                    quant1 a = quantize_one(W[o * I + i], sj, zb, qmax);
                    double cs, cz, cw;
                    if (a.side == 0)      { cs = a.r - (double)a.t; cz = 0.0;         cw = 1.0; }
                    else if (a.side < 0)  { cs = -zb;               cz = -(double)sj; cw = 0.0; }
                    else                  { cs = qmax - zb;         cz = -(double)sj; cw = 0.0; }
                    gs += acc[i] * cs;
                    gz += acc[i] * cz;
                    if (dW) dW[o * I + i] = acc[i] * cw;
                }
                if (ds) ds[o * G + j] = gs;
                if (dz) dz[o * G + j] = gz;
            }
        }
        free(acc);
    }
    return fail ? -2 : 0;
}

/* ---- storage format after Block-AP (Sec. 3.2 last paragraph, App. E) ------
 * W_q and z at N bits, s separately.  The paper fixes no bit layout; this one
 * is ours: each row is a little-endian bit stream, code i of the row occupying
 * bits [i*N, (i+1)*N); the stream is stored as bytes, least significant first.
 * Row stride of W_q: I*N/8 bytes (I % 32 == 0 keeps rows on 32-bit words for
 * every N).  Row stride of z: 4*ceil(G*N/32) bytes, tail bits zero.           */
i64 eqo_packed_w_row_bytes(i64 I, int bits) { return I * bits / 8; }
i64 eqo_packed_z_row_bytes(i64 G, int bits) { return 4 * ((G * bits + 31) / 32); }

static void put_bits(uint8_t *row, i64 idx, int bits, unsigned v)
{
    for (int b = 0; b < bits; ++b) {
        const i64 pos = idx * bits + b;
        if ((v >> b) & 1u) row[pos >> 3] |= (uint8_t)(1u << (pos & 7));
    }
}

static unsigned get_bits(const uint8_t *row, i64 idx, int bits)
{
    unsigned v = 0;
    for (int b = 0; b < bits; ++b) {
        const i64 pos = idx * bits + b;
        v |= (unsigned)((row[pos >> 3] >> (pos & 7)) & 1u) << b;
    }
    return v;
}

int eqo_pack(const float *W, const float *s, const float *z, i64 O, i64 I, int bits, i64 g,
             uint8_t *Wpacked, uint8_t *zpacked)
{
    if (!W || !s || !z || !Wpacked || !zpacked || bad_shape(I, O, bits, g) || I % 32 != 0) return -1;
    const i64 G = I / g;
    const double qmax = (double)((1 << bits) - 1);
    const i64 wrb = eqo_packed_w_row_bytes(I, bits), zrb = eqo_packed_z_row_bytes(G, bits);
#pragma omp parallel for schedule(static)
    for (i64 o = 0; o < O; ++o) {
        uint8_t *wr = Wpacked + o * wrb, *zr = zpacked + o * zrb;
        memset(wr, 0, (size_t)wrb);
        memset(zr, 0, (size_t)zrb);
        for (i64 j = 0; j < G; ++j) {
            const double zb = zbar_of(z[o * G + j], qmax);      /* in [0, Qmax]: the zero point Block-AP used */
            put_bits(zr, j, bits, (unsigned)zb);
            for (i64 i = j * g; i < (j + 1) * g; ++i) {
                quant1 a = quantize_one(W[o * I + i], s[o * G + j], zb, qmax);
                put_bits(wr, i, bits, (unsigned)a.q);
            }
        }
    }
    return 0;
}

int eqo_unpack(const uint8_t *Wpacked, const uint8_t *zpacked, i64 O, i64 I, int bits, i64 g,
               int32_t *codes, int32_t *zcodes)
{
    if (!Wpacked || !zpacked || bad_shape(I, O, bits, g) || I % 32 != 0) return -1;
    const i64 G = I / g;
    const i64 wrb = eqo_packed_w_row_bytes(I, bits), zrb = eqo_packed_z_row_bytes(G, bits);
#pragma omp parallel for schedule(static)
    for (i64 o = 0; o < O; ++o) {
        if (codes)
            for (i64 i = 0; i < I; ++i) codes[o * I + i] = (int32_t)get_bits(Wpacked + o * wrb, i, bits);
        if (zcodes)
            for (i64 j = 0; j < G; ++j) zcodes[o * G + j] = (int32_t)get_bits(zpacked + o * zrb, j, bits);
    }
    return 0;
}

/* ---- E2E-QP (Sec. 3.3): codes frozen, only Eq.(2) runs --------------------
 *   What = (w_q - z) * s,   Y = X * What^T
 *   dX = dY * What,  ds[o,j] = sum_{i in j} (dY^T X)[o,i] * (w_q[o,i] - z[o,j]) */
static void dequant_packed_row(const uint8_t *wr, const uint8_t *zr, const float *srow, i64 I, i64 g,
                               int bits, double *out)
{
    for (i64 i = 0; i < I; ++i) {
        const i64 j = i / g;
        const double q = (double)get_bits(wr, i, bits), zq = (double)get_bits(zr, j, bits);
        out[i] = (q - zq) * (double)srow[j];
    }
}

int eqo_qlinear_fwd(const float *X, const uint8_t *Wpacked, const float *s, const uint8_t *zpacked,
                    i64 T, i64 I, i64 O, int bits, i64 g, double *Y)
{
    if (!Wpacked || !s || !zpacked || bad_shape(I, O, bits, g) || I % 32 != 0 || T < 0) return -1;
    if (T == 0) return 0;
    if (!X || !Y) return -1;
    const i64 G = I / g;
    const i64 wrb = eqo_packed_w_row_bytes(I, bits), zrb = eqo_packed_z_row_bytes(G, bits);
    int fail = 0;
#pragma omp parallel
    {
        double *wh = (double *)malloc((size_t)I * sizeof(double));
        if (!wh) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (i64 o = 0; o < O; ++o) {
            if (!wh) continue;
            dequant_packed_row(Wpacked + o * wrb, zpacked + o * zrb, s + o * G, I, g, bits, wh);
            for (i64 t = 0; t < T; ++t) {
                const float *x = X + t * I;
                double acc = 0.0;
                for (i64 i = 0; i < I; ++i) acc += (double)x[i] * wh[i];
                Y[t * O + o] = acc;
            }
        }
        free(wh);
    }
    return fail ? -2 : 0;
}

int eqo_qlinear_bwd(const float *X, const uint8_t *Wpacked, const float *s, const uint8_t *zpacked,
                    const float *dY, i64 T, i64 I, i64 O, int bits, i64 g, double *dX, double *ds)
{
    if (!Wpacked || !s || !zpacked || bad_shape(I, O, bits, g) || I % 32 != 0 || T < 0) return -1;
    if (T > 0 && !dY) return -1;
    if (ds && T > 0 && !X) return -1;
    const i64 G = I / g;
    const i64 wrb = eqo_packed_w_row_bytes(I, bits), zrb = eqo_packed_z_row_bytes(G, bits);

    if (dX && T > 0) {
        double *What = (double *)malloc((size_t)O * (size_t)I * sizeof(double));
        if (!What) return -2;
#pragma omp parallel for schedule(static)
        for (i64 o = 0; o < O; ++o)
            dequant_packed_row(Wpacked + o * wrb, zpacked + o * zrb, s + o * G, I, g, bits, What + o * I);
        dx_from_what(dY, What, T, I, O, dX);
        free(What);
    }
    if (!ds) return 0;

    int fail = 0;
#pragma omp parallel
    {
        double *acc = (double *)malloc((size_t)I * sizeof(double));
        if (!acc) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (i64 o = 0; o < O; ++o) {
            if (!acc) continue;
            dwhat_row(X, dY, T, I, O, o, acc);
            for (i64 j = 0; j < G; ++j) {
                const double zq = (double)get_bits(zpacked + o * zrb, j, bits);
                double gs = 0.0;
                for (i64 i = j * g; i < (j + 1) * g; ++i)
                    gs += acc[i] * ((double)get_bits(Wpacked + o * wrb, i, bits) - zq);
                ds[o * G + j] = gs;
            }
        }
        free(acc);
    }
    return fail ? -2 : 0;
}

/* ---- E2E-QP with trainable zero points (Sec. 3.3; ablation "trainable parameters of E2E-QP") -----------------
 * When z is trained end to end it leaves its N-bit storage and becomes a floating-point tensor (the ablation's
 * average bit count rises from N + 16/g (+N/g) to N + 32/g for that reason).  There is no Eq.(1) in this phase,
 * so z enters Eq.(2) as it is, without rounding:
 *   What[o,i] = (w_q[o,i] - z[o,j]) * s[o,j],            Y = X * What^T,     dX = dY * What,
 *   ds[o,j] = sum_{i in j} dWhat[o,i] * (w_q[o,i] - z[o,j]),
 *   dz[o,j] = sum_{i in j} dWhat[o,i] * (-s[o,j])         (derivative of Eq.(2) with respect to z),
 * with dWhat = dY^T X. */
static void dequant_packed_row_fz(const uint8_t *wr, const float *zrow, const float *srow, i64 I, i64 g,
                                  int bits, double *out)
{
    for (i64 i = 0; i < I; ++i) {
        const i64 j = i / g;
        out[i] = ((double)get_bits(wr, i, bits) - (double)zrow[j]) * (double)srow[j];
    }
}

int eqo_qlinear_fwd_z(const float *X, const uint8_t *Wpacked, const float *s, const float *z,
                      i64 T, i64 I, i64 O, int bits, i64 g, double *Y)
{
    if (!Wpacked || !s || !z || bad_shape(I, O, bits, g) || I % 32 != 0 || T < 0) return -1;
    if (T == 0) return 0;
    if (!X || !Y) return -1;
    const i64 G = I / g;
    const i64 wrb = eqo_packed_w_row_bytes(I, bits);
    int fail = 0;
#pragma omp parallel
    {
        double *wh = (double *)malloc((size_t)I * sizeof(double));
        if (!wh) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (i64 o = 0; o < O; ++o) {
            if (!wh) continue;
            dequant_packed_row_fz(Wpacked + o * wrb, z + o * G, s + o * G, I, g, bits, wh);
            for (i64 t = 0; t < T; ++t) {
                const float *x = X + t * I;
                double acc = 0.0;
                for (i64 i = 0; i < I; ++i) acc += (double)x[i] * wh[i];
                Y[t * O + o] = acc;
            }
        }
        free(wh);
    }
    return fail ? -2 : 0;
}

int eqo_qlinear_bwd_z(const float *X, const uint8_t *Wpacked, const float *s, const float *z,
                      const float *dY, i64 T, i64 I, i64 O, int bits, i64 g, double *dX, double *ds, double *dz)
{
    if (!Wpacked || !s || !z || bad_shape(I, O, bits, g) || I % 32 != 0 || T < 0) return -1;
    if (T > 0 && !dY) return -1;
    if ((ds || dz) && T > 0 && !X) return -1;
    const i64 G = I / g;
    const i64 wrb = eqo_packed_w_row_bytes(I, bits);

    if (dX && T > 0) {
        double *What = (double *)malloc((size_t)O * (size_t)I * sizeof(double));
        if (!What) return -2;
#pragma omp parallel for schedule(static)
        for (i64 o = 0; o < O; ++o)
            dequant_packed_row_fz(Wpacked + o * wrb, z + o * G, s + o * G, I, g, bits, What + o * I);
        dx_from_what(dY, What, T, I, O, dX);
        free(What);
    }
    if (!ds && !dz) return 0;

    int fail = 0;
#pragma omp parallel
    {
        double *acc = (double *)malloc((size_t)I * sizeof(double));
        if (!acc) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (i64 o = 0; o < O; ++o) {
            if (!acc) continue;
            dwhat_row(X, dY, T, I, O, o, acc);
            for (i64 j = 0; j < G; ++j) {
                const double zf = (double)z[o * G + j], sf = (double)s[o * G + j];
                double gs = 0.0, gz = 0.0;
                for (i64 i = j * g; i < (j + 1) * g; ++i) {
                    gs += acc[i] * ((double)get_bits(Wpacked + o * wrb, i, bits) - zf);
                    gz += acc[i] * (-sf);
                }
                if (ds) ds[o * G + j] = gs;
                if (dz) dz[o * G + j] = gz;
            }
        }
        free(acc);
    }
    return fail ? -2 : 0;
}

/* ------------------------------------------------------------------------------------------------------------------
 * Block-AP step glue (Sec. 3.2: a block is trained against the output of its full-precision counterpart with a
 * reconstruction loss; Sec. 4.1 "Training": one learning rate for the quantization parameters, another for the weights).
 * The paper names neither the form of the loss nor the optimizer.  Taken here: the mean squared error over all elements
 * of the block output, and AdamW (Adam with bias correction and decoupled weight decay) as published by its authors.
 * ------------------------------------------------------------------------------------------------------------------ */

/* loss = (1/n) * sum (Y - Yref)^2 ;  dY = d loss / d Y = 2 (Y - Yref) / n.   dY may be NULL. */
int eqo_recon_loss(const float *Y, const float *Yref, i64 n, double *loss, double *dY)
{
    if (n < 1 || !Y || !Yref || !loss) return -1;
    double acc = 0.0;
    for (i64 k = 0; k < n; ++k) {
        const double e = (double)Y[k] - (double)Yref[k];
        acc += e * e;
        if (dY) dY[k] = 2.0 * e / (double)n;
    }
    *loss = acc / (double)n;
    return 0;
}

/* One AdamW step on n parameters, in place (p, m, v), `step` counted from 1:
 *   p <- p - lr * wd * p
 *   m <- b1 m + (1 - b1) g ;  v <- b2 v + (1 - b2) g^2
 *   p <- p - lr * (m / (1 - b1^step)) / (sqrt(v / (1 - b2^step)) + eps)
 *   p <- max(p, p_min)
 * p_min: the step sizes are held at or above the 1e-10 of their initialisation (Eq.(1) divides by s: the paper's method
 * needs s > 0 and has nothing that keeps an optimizer step from crossing zero); -inf for parameters without a bound.   */
int eqo_adamw(double *p, const float *grad, double *m, double *v, i64 n,
              double lr, double b1, double b2, double eps, double wd, int step, double p_min)
{
    if (n < 0 || step < 1 || (n > 0 && (!p || !grad || !m || !v))) return -1;
    const double c1 = 1.0 - pow(b1, (double)step), c2 = 1.0 - pow(b2, (double)step);
    for (i64 k = 0; k < n; ++k) {
        const double gk = (double)grad[k];
        p[k] -= lr * wd * p[k];
        m[k] = b1 * m[k] + (1.0 - b1) * gk;
        v[k] = b2 * v[k] + (1.0 - b2) * gk * gk;
        p[k] -= lr * (m[k] / c1) / (sqrt(v[k] / c2) + eps);
        if (p[k] < p_min) p[k] = p_min;
    }
    return 0;
}
