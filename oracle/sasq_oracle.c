/*
 * SASQ CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, scalar implementation of the SASQ hot path written directly
 * from the paper's definitions.  It exists only so that tests, the smoke check
 * and the benchmark's cpu_baseline leg have something independent to compare
 * the HIP library against.  It shares no source, header, table or helper with
 * the HIP path and must never be called from it.
 *
 * What it follows:
 *   - symmetric N-bit quantizer  X_int = clamp(round(X/S), -2^(N-1), 2^(N-1)-1),
 *     absmax scale S = max|X| / (2^(N-1)-1)                     (Sec. 3, Eq. 1)
 *   - fake quantization = quant, round, clamp, dequant: X' = S_x * X_int
 *                                                    (Sec. 4.2; Sec. 4.3, Eq. 5)
 *   - straight-through estimator: d round/dx = 1, d clamp/dx = 1 inside
 *     [min,max] and 0 outside                                   (Sec. 4.2, Eq. 4)
 *   - quantized linear  Y = S_x * (X_int . W_int) * S_w, integer product first,
 *     then inverse quantization, bias left unquantized          (Sec. 3, Eq. 2)
 *   - static quantization: S_x is a fixed input, never recomputed from X
 *                                                    (Sec. 3; Sec. 4.5; Fig. 1)
 *
 * Readings where the paper gives only a real-number formula (all are listed
 * again in the design notes of the repository):
 *   - round() is round-half-to-even of the exact product x * inv_s with
 *     inv_s = fl32(1/s); the product of a 16-bit float and an fp32 is exact
 *     in fp64, so rint((double)x * (double)inv_s) is that value.
 *   - the clamp indicator of the STE is taken on clamp's own argument, i.e. on
 *     the rounded value r, bounds inclusive.
 *   - gradient of the scale, from the chain rule with Eq. 4 and dv/ds = -v/s:
 *         d x'/d s = q - m*v,   ds = sum_i dy_i * (q_i - m_i * v_i).
 *   - dequantization is one fp32 multiply followed by one round-to-nearest-even
 *     conversion to the 16-bit storage type; the linear's epilogue is
 *     c[n] = fl32(s * s_w[n]), y = fl32(fl32(acc) * c[n]) (+ bias in fp32).
 *   - int4 weights: two's-complement nibbles, element k even in the low nibble.
 *
 * Parity pins: every function here is pinned by tests that do not go through
 * this file's own formulas (hand table, exact rational arithmetic, autograd,
 * int64 matmul, library float conversions); none is "parity unpinned".
 */
#include <fenv.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { DT_F16 = 0, DT_BF16 = 1 };
enum { WF_INT8 = 0, WF_INT4_PACKED = 1 };
enum { FLAG_NO_ROUND = 1, FLAG_NO_CLAMP = 2, FLAG_STE_ON_V = 4 };
enum { OK = 0, ERR_ARG = 1, ERR_ROUNDING_MODE = 2, ERR_NOMEM = 3 };

/* ---- 16-bit storage formats, written from the IEEE-754 / bfloat16 layouts ---- */

/* binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static double f16_to_double(uint16_t h)
{
    int sign = h >> 15, e = (h >> 10) & 0x1F, f = h & 0x3FF;
    double v;
    if (e == 0)        v = ldexp((double)f, -24);              /* subnormal: f * 2^-24 */
    else if (e == 31)  v = f ? NAN : INFINITY;
    else               v = ldexp((double)(1024 + f), e - 25);  /* (1 + f/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* bfloat16: 1 sign, 8 exponent (bias 127), 7 fraction bits. */
static double bf16_to_double(uint16_t b)
{
    int sign = b >> 15, e = (b >> 7) & 0xFF, f = b & 0x7F;
    double v;
    if (e == 0)        v = ldexp((double)f, -133);             /* f * 2^-7 * 2^-126 */
    else if (e == 255) v = f ? NAN : INFINITY;
    else               v = ldexp((double)(128 + f), e - 134);  /* (1 + f/128) * 2^(e-127) */
    return sign ? -v : v;
}

/* Round a real value to a format with `fbits` fraction bits, exponent bias `bias`
 * and `ebits` exponent bits, nearest-even, overflow to infinity. */
static uint16_t round_to_small_float(double v, int fbits, int ebits, int bias)
{
    uint16_t sign = signbit(v) ? (uint16_t)(1u << (fbits + ebits)) : 0;
    int emax_field = (1 << ebits) - 1;
    double a = fabs(v);
    if (isnan(a)) return (uint16_t)(sign | (emax_field << fbits) | 1);
    if (isinf(a)) return (uint16_t)(sign | (emax_field << fbits));
    if (a == 0.0) return sign;
    int emin = 1 - bias;                        /* exponent of the smallest normal */
    int ex;
    (void)frexp(a, &ex);                        /* a = fr * 2^ex, fr in [0.5,1) */
    int e = ex - 1;                             /* a in [2^e, 2^(e+1)) */
    if (e < emin) {                             /* subnormal spacing 2^(emin-fbits) */
        double m = rint(ldexp(a, fbits - emin));
        return (uint16_t)(sign | (uint16_t)m);  /* m == 2^fbits lands on the smallest normal */
    }
    double m = rint(ldexp(a, fbits - e));       /* in [2^fbits, 2^(fbits+1)] */
    if (m == ldexp(1.0, fbits + 1)) { m = ldexp(1.0, fbits); e += 1; }
    int field = e + bias;
    if (field >= emax_field) return (uint16_t)(sign | (emax_field << fbits));
    return (uint16_t)(sign | (field << fbits) | ((int)m - (1 << fbits)));
}

static uint16_t f32_to_f16(float f)  { return round_to_small_float((double)f, 10, 5, 15); }
static uint16_t f32_to_bf16(float f) { return round_to_small_float((double)f, 7, 8, 127); }

static double load16(const uint16_t* p, int64_t i, int dt)
{
    return dt == DT_F16 ? f16_to_double(p[i]) : bf16_to_double(p[i]);
}
static uint16_t store16(float f, int dt) { return dt == DT_F16 ? f32_to_f16(f) : f32_to_bf16(f); }

/* exported for the tests that pin the converters against library routines */
void sasq_oracle_decode16(const uint16_t* in, double* out, int64_t n, int dt)
{
    for (int64_t i = 0; i < n; ++i) out[i] = load16(in, i, dt);
}
void sasq_oracle_encode16(const float* in, uint16_t* out, int64_t n, int dt)
{
    for (int64_t i = 0; i < n; ++i) out[i] = store16(in[i], dt);
}

int sasq_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- the quantizer (Sec. 3, Eq. 1) with the STE indicator (Sec. 4.2, Eq. 4) ---- */

typedef struct {
    double p;   /* v = x / s, evaluated as the exact product x * inv_s          */
    double r;   /* round(v), ties to even (or v itself with FLAG_NO_ROUND)      */
    double q;   /* clamp(r, Qn, Qp): the integer code (unbounded with NO_CLAMP) */
    int    m;   /* 1 if clamp passes its argument through, else 0               */
} qelem;

static qelem quantize_one(double x, float inv_s, int Qn, int Qp, int flags)
{
    qelem e;
    e.p = x * (double)inv_s;
    e.r = (flags & FLAG_NO_ROUND) ? e.p : rint(e.p);
    if (flags & FLAG_NO_CLAMP) { e.m = 1; e.q = e.r; return e; }
    double u = (flags & FLAG_STE_ON_V) ? e.p : e.r;
    e.m = (u >= (double)Qn && u <= (double)Qp) ? 1 : 0;
    e.q = e.r < (double)Qn ? (double)Qn : (e.r > (double)Qp ? (double)Qp : e.r);
    return e;
}

static int check_common(int bits, int dt)
{
    if (bits < 2 || bits > 8) return ERR_ARG;
    if (dt != DT_F16 && dt != DT_BF16) return ERR_ARG;
    if (fegetround() != FE_TONEAREST) return ERR_ROUNDING_MODE;
    return OK;
}

/* fl32(1/s): one correctly rounded fp32 division. */
static float reciprocal_f32(float s)
{
    volatile float one = 1.0f, d = s;
    volatile float r = one / d;
    return r;
}

float sasq_oracle_inv_scale(float s) { return reciprocal_f32(s); }

/*
 * Fake-quant forward: y = s * clamp(round(x/s), Qn, Qp)  (Sec. 4.2; Eq. 1; Eq. 5).
 * x, y: [rows, cols] 16-bit patterns; codes (optional): int8; v_out, r_out (optional): fp64.
 */
int sasq_oracle_fakequant_fwd(const uint16_t* x, float s, uint16_t* y, int8_t* codes,
                              int64_t rows, int64_t cols, int bits, int dt, int flags)
{
    int rc = check_common(bits, dt);
    if (rc) return rc;
    const int Qn = -(1 << (bits - 1)), Qp = (1 << (bits - 1)) - 1;
    const float inv_s = reciprocal_f32(s);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t j = 0; j < cols; ++j) {
            int64_t idx = i * cols + j;
            qelem e = quantize_one(load16(x, idx, dt), inv_s, Qn, Qp, flags);
            volatile float qf = (float)e.q;      /* exact for integer codes */
            volatile float yf = qf * s;          /* one fp32 multiply */
            if (y) y[idx] = store16(yf, dt);
            if (codes) codes[idx] = (int8_t)e.q;
        }
    }
    return OK;
}

/*
 * Fake-quant backward (Sec. 4.2, Eq. 4 + chain rule):
 *   dx = dy * m                      (bit pattern of dy, or +0)
 *   ds = sum dy * (q - m*v)          fp64 per row, rows summed in order, rounded once to fp32.
 * Optional outputs: ds64 (the fp64 sum), sum_abs (sum |dy*(q-m*v)|, for conditioning).
 */
int sasq_oracle_fakequant_bwd(const uint16_t* x, const uint16_t* dy, float s, uint16_t* dx,
                              float* ds, double* ds64, double* sum_abs,
                              int64_t rows, int64_t cols, int bits, int dt, int flags)
{
    int rc = check_common(bits, dt);
    if (rc) return rc;
    const int Qn = -(1 << (bits - 1)), Qp = (1 << (bits - 1)) - 1;
    const float inv_s = reciprocal_f32(s);
    double* row_sum = (double*)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1) * 2);
    if (!row_sum) return ERR_NOMEM;
    double* row_abs = row_sum + (rows > 0 ? rows : 1);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        double acc = 0.0, aabs = 0.0;
        for (int64_t j = 0; j < cols; ++j) {
            int64_t idx = i * cols + j;
            qelem e = quantize_one(load16(x, idx, dt), inv_s, Qn, Qp, flags);
            double g = load16(dy, idx, dt);
            if (dx) dx[idx] = e.m ? dy[idx] : (uint16_t)0;
            double t;
            if (e.m) t = isinf(e.p) ? 0.0 : g * (e.q - e.p);   /* only NO_CLAMP reaches the inf guard */
            else     t = g * e.q;
            acc += t;
            aabs += fabs(t);
        }
        row_sum[i] = acc;
        row_abs[i] = aabs;
    }
    double total = 0.0, total_abs = 0.0;
    for (int64_t i = 0; i < rows; ++i) { total += row_sum[i]; total_abs += row_abs[i]; }
    free(row_sum);
    if (ds) *ds = (float)total;
    if (ds64) *ds64 = total;
    if (sum_abs) *sum_abs = total_abs;
    return OK;
}

/* Sign-extend the two's-complement nibble (Sec. 3, Eq. 1 with N = 4 gives [-8, 7]). */
static int nibble_to_int(unsigned v) { return (v & 8u) ? (int)v - 16 : (int)v; }

/*
 * Static-inference quantized linear (Sec. 3, Eq. 2; static scale: Sec. 3, Sec. 4.5):
 *   xq[m,k]  = clamp(round(x[m,k]/s), Qn, Qp)
 *   acc[m,n] = sum_k xq[m,k] * Wq[n,k]                  exact int32
 *   Y[m,n]   = fl32(fl32(acc) * fl32(s * s_w[n])) (+ bias[n] in fp32) -> 16-bit RNE
 * wq: [N,K] int8, or [N,K/2] bytes of packed int4 (k even -> low nibble).
 */
int sasq_oracle_static_linear(const uint16_t* x, float s, const uint8_t* wq, const float* s_w,
                              const float* bias, uint16_t* y, int32_t* acc_out, int8_t* xq_out,
                              int64_t M, int64_t N, int64_t K, int a_bits, int wf, int dt)
{
    int rc = check_common(a_bits, dt);
    if (rc) return rc;
    if (wf != WF_INT8 && wf != WF_INT4_PACKED) return ERR_ARG;
    if (wf == WF_INT4_PACKED && (K & 1)) return ERR_ARG;
    const int Qn = -(1 << (a_bits - 1)), Qp = (1 << (a_bits - 1)) - 1;
    const float inv_s = reciprocal_f32(s);

    int8_t* xq = (int8_t*)malloc((size_t)(M * K > 0 ? M * K : 1));
    int8_t* w8 = (int8_t*)malloc((size_t)(N * K > 0 ? N * K : 1));
    if (!xq || !w8) { free(xq); free(w8); return ERR_NOMEM; }

#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            xq[m * K + k] = (int8_t)quantize_one(load16(x, m * K + k, dt), inv_s, Qn, Qp, 0).q;
    if (xq_out) memcpy(xq_out, xq, (size_t)(M * K));

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            if (wf == WF_INT8) w8[n * K + k] = (int8_t)wq[n * K + k];
            else {
                uint8_t byte = wq[n * (K / 2) + k / 2];
                w8[n * K + k] = (int8_t)nibble_to_int((k & 1) ? (byte >> 4) : (byte & 15u));
            }
        }

#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int32_t)xq[m * K + k] * (int32_t)w8[n * K + k];
            if (acc_out) acc_out[m * N + n] = acc;
            if (y) {
                volatile float c = s * s_w[n];
                volatile float af = (float)acc;
                volatile float yf = af * c;
                if (bias) { volatile float yb = yf + bias[n]; yf = yb; }
                y[m * N + n] = store16(yf, dt);
            }
        }
    }
    free(xq);
    free(w8);
    return OK;
}

/*
 * Static linear with one activation factor per group of `group` consecutive input channels
 * (Sec. 3, Eq. 3: Y = sum_i (S_x,i * S_w) * (X_int,i . W_int), the block-wise form the paper gives
 * for activations quantized per channel; Sec. 4 uses per-channel activation factors).  Each
 * channel k is quantized with s_g[k / group] (Eq. 1); each group's integer product is exact in
 * int32; the groups are accumulated in fp32 in ascending order with one fused multiply-add per
 * group (reading: Eq. 3 fixes no rounding order), the per-output-channel weight factor and the
 * bias are applied last:
 *     f = 0;  for i in 0..G-1:  f = fma(fl32(acc_i), s_g[i], f);   Y = fl32(f * s_w[n]) (+ bias[n]).
 * group = 1 is per-channel in the strict sense, group = K per-tensor (with this rounding order).
 * f_out (optional) receives f, xq_out the codes.
 */
int sasq_oracle_static_linear_grouped(const uint16_t* x, const float* s_g, const uint8_t* wq, const float* s_w,
                                      const float* bias, uint16_t* y, float* f_out, int8_t* xq_out,
                                      int64_t M, int64_t N, int64_t K, int64_t group, int a_bits, int wf, int dt)
{
    int rc = check_common(a_bits, dt);
    if (rc) return rc;
    if (wf != WF_INT8 && wf != WF_INT4_PACKED) return ERR_ARG;
    if (wf == WF_INT4_PACKED && (K & 1)) return ERR_ARG;
    if (group <= 0 || K % group) return ERR_ARG;
    const int64_t G = K / group;
    const int Qn = -(1 << (a_bits - 1)), Qp = (1 << (a_bits - 1)) - 1;

    int8_t* xq = (int8_t*)malloc((size_t)(M * K > 0 ? M * K : 1));
    int8_t* w8 = (int8_t*)malloc((size_t)(N * K > 0 ? N * K : 1));
    if (!xq || !w8) { free(xq); free(w8); return ERR_NOMEM; }

#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            xq[m * K + k] = (int8_t)quantize_one(load16(x, m * K + k, dt), reciprocal_f32(s_g[k / group]), Qn, Qp, 0).q;
    if (xq_out) memcpy(xq_out, xq, (size_t)(M * K));

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            if (wf == WF_INT8) w8[n * K + k] = (int8_t)wq[n * K + k];
            else {
                uint8_t byte = wq[n * (K / 2) + k / 2];
                w8[n * K + k] = (int8_t)nibble_to_int((k & 1) ? (byte >> 4) : (byte & 15u));
            }
        }

#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            float f = 0.0f;
            for (int64_t i = 0; i < G; ++i) {
                int32_t acc = 0;
                for (int64_t k = i * group; k < (i + 1) * group; ++k)
                    acc += (int32_t)xq[m * K + k] * (int32_t)w8[n * K + k];
                f = fmaf((float)acc, s_g[i], f);
            }
            if (f_out) f_out[m * N + n] = f;
            if (y) {
                volatile float yf = f * s_w[n];
                if (bias) { volatile float yb = yf + bias[n]; yf = yb; }
                y[m * N + n] = store16(yf, dt);
            }
        }
    }
    free(xq);
    free(w8);
    return OK;
}

/*
 * Dynamic per-token linear: the baseline the paper's static factors replace (Sec. 3: dynamic
 * quantization computes the factors during inference; per-token = one factor per row of X,
 * Fig. 2(b); Sec. 4.5 compares against it).  For every row m:
 *     s_m      = fl32(max_k |X[m,k]| / Qp)          (Eq. 1's S on the row; 1 if the row is all zero)
 *     xq[m,k]  = clamp(RHE(X[m,k] * fl32(1/s_m)))    (Eq. 1)
 *     acc[m,n] = sum_k xq[m,k] * Wq[n,k]             (exact int32)
 *     Y[m,n]   = fl32(fl32(acc) * fl32(s_m * s_w[n])) (+ bias[n])       (Eq. 2 with S_x per row)
 * Inputs must be finite.  s_row_out (optional) receives the M factors.
 */
int sasq_oracle_dynamic_linear(const uint16_t* x, const uint8_t* wq, const float* s_w, const float* bias,
                               uint16_t* y, int32_t* acc_out, int8_t* xq_out, float* s_row_out,
                               int64_t M, int64_t N, int64_t K, int a_bits, int wf, int dt)
{
    int rc = check_common(a_bits, dt);
    if (rc) return rc;
    if (wf != WF_INT8 && wf != WF_INT4_PACKED) return ERR_ARG;
    if (wf == WF_INT4_PACKED && (K & 1)) return ERR_ARG;
    const int Qn = -(1 << (a_bits - 1)), Qp = (1 << (a_bits - 1)) - 1;

    int8_t* xq = (int8_t*)malloc((size_t)(M * K > 0 ? M * K : 1));
    int8_t* w8 = (int8_t*)malloc((size_t)(N * K > 0 ? N * K : 1));
    float* srow = (float*)malloc(sizeof(float) * (size_t)(M > 0 ? M : 1));
    if (!xq || !w8 || !srow) { free(xq); free(w8); free(srow); return ERR_NOMEM; }

#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double amax = 0.0;
        for (int64_t k = 0; k < K; ++k) { double a = fabs(load16(x, m * K + k, dt)); if (a > amax) amax = a; }
        volatile float num = (float)amax;            /* exact: a 16-bit float */
        volatile float den = (float)Qp;
        volatile float sm = num / den;
        if (amax == 0.0) sm = 1.0f;
        srow[m] = sm;
        const float inv = reciprocal_f32(sm);
        for (int64_t k = 0; k < K; ++k)
            xq[m * K + k] = (int8_t)quantize_one(load16(x, m * K + k, dt), inv, Qn, Qp, 0).q;
    }
    if (xq_out) memcpy(xq_out, xq, (size_t)(M * K));
    if (s_row_out) memcpy(s_row_out, srow, sizeof(float) * (size_t)M);

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            if (wf == WF_INT8) w8[n * K + k] = (int8_t)wq[n * K + k];
            else {
                uint8_t byte = wq[n * (K / 2) + k / 2];
                w8[n * K + k] = (int8_t)nibble_to_int((k & 1) ? (byte >> 4) : (byte & 15u));
            }
        }

#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int32_t)xq[m * K + k] * (int32_t)w8[n * K + k];
            if (acc_out) acc_out[m * N + n] = acc;
            if (y) {
                volatile float c = srow[m] * s_w[n];
                volatile float af = (float)acc;
                volatile float yf = af * c;
                if (bias) { volatile float yb = yf + bias[n]; yf = yb; }
                y[m * N + n] = store16(yf, dt);
            }
        }
    }
    free(xq);
    free(w8);
    free(srow);
    return OK;
}

/*
 * Backward of the training-time linear with respect to its (fake-quantized) input: the step that
 * hands the fake-quant operator its upstream gradient during scale training (Sec. 4.2: gradients
 * flow back through the frozen, quantized linear layers to the quantization factors).  The frozen
 * weight takes part as the dequantized tensor held in the model's 16-bit type (Eq. 2's
 * W_int * S_w, one factor per output channel; reading: rounded once to the storage type, as a
 * framework holding the fake-quantized weight would):
 *     Wq[n,k]  = round16(fl32(fl32(W_int[n,k]) * s_w[n]))
 *     dX[m,k]  = round16(sum_n dY[m,n] * Wq[n,k])        (sum in fp64 here; products are exact)
 * wq16_out (optional) receives Wq as 16-bit patterns, sum_abs_out (optional) sum_n |dY*Wq| per
 * output (the scale of the fp32 accumulation error a GPU kernel is allowed).
 */
int sasq_oracle_linear_bwd_input(const uint16_t* dy, const uint8_t* wq, const float* s_w, uint16_t* dx,
                                 uint16_t* wq16_out, double* sum_abs_out, double* exact_out,
                                 int64_t M, int64_t N, int64_t K, int wf, int dt)
{
    if (dt != DT_F16 && dt != DT_BF16) return ERR_ARG;
    if (wf != WF_INT8 && wf != WF_INT4_PACKED) return ERR_ARG;
    if (wf == WF_INT4_PACKED && (K & 1)) return ERR_ARG;
    uint16_t* w16 = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)(N * K > 0 ? N * K : 1));
    if (!w16) return ERR_NOMEM;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            int w;
            if (wf == WF_INT8) w = (int8_t)wq[n * K + k];
            else {
                uint8_t byte = wq[n * (K / 2) + k / 2];
                w = nibble_to_int((k & 1) ? (byte >> 4) : (byte & 15u));
            }
            volatile float wf32 = (float)w;
            volatile float prod = wf32 * s_w[n];
            w16[n * K + k] = store16(prod, dt);
        }
    if (wq16_out) memcpy(wq16_out, w16, sizeof(uint16_t) * (size_t)(N * K));
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            double acc = 0.0, sabs = 0.0;
            for (int64_t n = 0; n < N; ++n) {
                const double t = load16(dy, m * N + n, dt) * load16(w16, n * K + k, dt);
                acc += t;
                sabs += fabs(t);
            }
            if (dx) dx[m * K + k] = store16((float)acc, dt);
            if (sum_abs_out) sum_abs_out[m * K + k] = sabs;
            if (exact_out) exact_out[m * K + k] = acc;
        }
    free(w16);
    return OK;
}

/*
 * Frozen-weight quantization, symmetric, one scale per output channel (row of W[N,K])
 * (Sec. 3, Eq. 1 applied per row; Sec. 5.1 fixes weights to one factor per output channel):
 *   s_w[n] = fl32(max_k |W[n,k]| / Qp)   (1 if the row is all zero)
 *   Wq[n,k] = clamp(round(W[n,k] / s_w[n]), Qn, Qp), round as for activations
 * bits = 8 -> int8 [N,K];  bits = 4 -> packed [N,K/2].
 */
int sasq_oracle_quantize_weight(const float* w, uint8_t* wq, float* s_w,
                                int64_t N, int64_t K, int wf)
{
    if (fegetround() != FE_TONEAREST) return ERR_ROUNDING_MODE;
    if (wf != WF_INT8 && wf != WF_INT4_PACKED) return ERR_ARG;
    if (wf == WF_INT4_PACKED && (K & 1)) return ERR_ARG;
    const int bits = wf == WF_INT8 ? 8 : 4;
    const int Qn = -(1 << (bits - 1)), Qp = (1 << (bits - 1)) - 1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) { float a = fabsf(w[n * K + k]); if (a > amax) amax = a; }
        volatile float sw = amax / (float)Qp;
        if (amax == 0.0f) sw = 1.0f;
        s_w[n] = sw;
        const float inv = reciprocal_f32(sw);
        for (int64_t k = 0; k < K; ++k) {
            int q = (int)quantize_one((double)w[n * K + k], inv, Qn, Qp, 0).q;
            if (wf == WF_INT8) wq[n * K + k] = (uint8_t)(int8_t)q;
            else {
                uint8_t* b = &wq[n * (K / 2) + k / 2];
                if (k & 1) *b = (uint8_t)((*b & 0x0F) | ((q & 15) << 4));
                else       *b = (uint8_t)((*b & 0xF0) | (q & 15));
            }
        }
    }
    return OK;
}

/* Absmax initial scale, S = max|X| / (2^(N-1) - 1)  (Sec. 3, Eq. 1 right half; Sec. 4.1). */
int sasq_oracle_absmax_scale(const uint16_t* x, float* s, int64_t n, int bits, int dt)
{
    int rc = check_common(bits, dt);
    if (rc) return rc;
    double amax = 0.0;
    for (int64_t i = 0; i < n; ++i) { double a = fabs(load16(x, i, dt)); if (a > amax) amax = a; }
    volatile float num = (float)amax;            /* exact: a 16-bit float */
    volatile float den = (float)((1 << (bits - 1)) - 1);
    volatile float r = num / den;
    *s = r;
    return OK;
}

/* Plain SGD on the scale, the only trained parameter (Sec. 4.2): s <- fl32(s - fl32(lr * ds)). */
float sasq_oracle_scale_sgd(float s, float ds, float lr)
{
    volatile float step = lr * ds;
    volatile float out = s - step;
    return out;
}

/*
 * Per-channel variants: one factor per activation column (Sec. 4: per-channel quantization for
 * activations; Sec. 2, Fig. 2(b): the elements of a column share a factor).  Element arithmetic
 * as above with s = s[k] for column k; the scale gradient is a sum over the rows of each column.
 */
int sasq_oracle_fakequant_fwd_pc(const uint16_t* x, const float* s, uint16_t* y, int8_t* codes,
                                 int64_t rows, int64_t cols, int bits, int dt)
{
    int rc = check_common(bits, dt);
    if (rc) return rc;
    const int Qn = -(1 << (bits - 1)), Qp = (1 << (bits - 1)) - 1;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < cols; ++k) {
        const float sk = s[k];
        const float inv_s = reciprocal_f32(sk);
        for (int64_t m = 0; m < rows; ++m) {
            int64_t idx = m * cols + k;
            qelem e = quantize_one(load16(x, idx, dt), inv_s, Qn, Qp, 0);
            volatile float qf = (float)e.q;
            volatile float yf = qf * sk;
            if (y) y[idx] = store16(yf, dt);
            if (codes) codes[idx] = (int8_t)e.q;
        }
    }
    return OK;
}

int sasq_oracle_fakequant_bwd_pc(const uint16_t* x, const uint16_t* dy, const float* s, uint16_t* dx,
                                 float* ds, double* ds64, double* sum_abs,
                                 int64_t rows, int64_t cols, int bits, int dt)
{
    int rc = check_common(bits, dt);
    if (rc) return rc;
    const int Qn = -(1 << (bits - 1)), Qp = (1 << (bits - 1)) - 1;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < cols; ++k) {
        const float inv_s = reciprocal_f32(s[k]);
        double acc = 0.0, aabs = 0.0;
        for (int64_t m = 0; m < rows; ++m) {
            int64_t idx = m * cols + k;
            qelem e = quantize_one(load16(x, idx, dt), inv_s, Qn, Qp, 0);
            double g = load16(dy, idx, dt);
            if (dx) dx[idx] = e.m ? dy[idx] : (uint16_t)0;
            double t = e.m ? g * (e.q - e.p) : g * e.q;
            acc += t;
            aabs += fabs(t);
        }
        if (ds) ds[k] = (float)acc;
        if (ds64) ds64[k] = acc;
        if (sum_abs) sum_abs[k] = aabs;
    }
    return OK;
}

/*
 * AdamW step on a vector of scales (the optimiser and learning rate of the paper's runs, Sec. 5.1
 * "Implementation"; the scales are the only parameters, Sec. 4.2).  Decoupled weight decay:
 *   p <- p - lr*wd*p;  m <- b1*m + (1-b1)*g;  v <- b2*v + (1-b2)*g^2;
 *   p <- p - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps).
 * Evaluated in fp64 on fp32 state; results rounded once to fp32.
 */
void sasq_oracle_scale_adamw(float* p, const float* g, float* m, float* v, int64_t n, int64_t step,
                             double lr, double b1, double b2, double eps, double wd)
{
    const double bc1 = 1.0 - pow(b1, (double)step), bc2 = 1.0 - pow(b2, (double)step);
    for (int64_t i = 0; i < n; ++i) {
        double pi = (double)p[i], gi = (double)g[i];
        pi -= lr * wd * pi;
        double mi = b1 * (double)m[i] + (1.0 - b1) * gi;
        double vi = b2 * (double)v[i] + (1.0 - b2) * gi * gi;
        pi -= lr * (mi / bc1) / (sqrt(vi / bc2) + eps);
        p[i] = (float)pi; m[i] = (float)mi; v[i] = (float)vi;
    }
}
