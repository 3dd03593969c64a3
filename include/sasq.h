/*
 * sasq.h -- C ABI of the SASQ hot-path library for AMD MI355X (gfx950).
 *
 * SASQ (Static Activation Scaling for Quantization-aware training) trains nothing but the
 * activation quantization factors of an LLM's linear layers and then runs those layers with
 * the trained factors held fixed.  This library is the data-parallel hot path of that method:
 *
 *   training:   x' = fakequant(x; s)                     sasq_fakequant_fwd
 *               dx, ds = backward(x, dy; s)              sasq_fakequant_bwd
 *               s <- s - lr * ds                         sasq_scale_sgd
 *   inference:  Y = s * (q(X) . Wq^T) * s_w (+ bias)     sasq_static_linear
 *   set-up:     Wq, s_w from frozen fp32 weights         sasq_quantize_weight
 *               s0 = max|X| / (2^(bits-1) - 1)           sasq_absmax_scale
 *
 * Conventions shared by every entry point
 *   - Every data pointer is DEVICE memory owned by the caller (the library never allocates,
 *     frees or keeps a pointer).  Scalars that are trained or produced on the device (s, ds)
 *     are device pointers too, so a training step needs no host synchronisation.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on that stream and return; outputs are valid once the stream has drained.
 *   - Matrices are dense row-major.  An activation matrix is [tokens, channels] (Sec. 2, Fig. 2).
 *   - 16-bit tensors are IEEE binary16 (SASQ_F16) or bfloat16 (SASQ_BF16).
 *   - Base pointers of 16-bit and weight tensors must be 16-byte aligned (SASQ_ERR_ALIGN).
 *   - Return value: a sasq_status.  Arguments are validated on the host before anything is
 *     launched; on error nothing has been enqueued.  The library never throws or aborts.
 *   - NOT validated (device-resident, checking would need a sync): *s finite and non-zero,
 *     inputs free of NaN.  Behaviour for such values is unspecified (but in-bounds).
 *   - Workspaces come from sasq_workspace_init(): a workspace is caller-owned device memory
 *     that must have been passed ONCE to sasq_workspace_init before its first use, may be reused
 *     by any number of later calls, and must not be used by two calls that can overlap in time.
 *   - Graph capture: an entry point only launches kernels on the caller's stream (no allocation,
 *     no copy, no memset, no synchronisation), so calls may be recorded into a HIP graph and
 *     replayed; items arrays and other host arguments are read before the call returns.
 *
 * Numerical contract (the paper gives real-number formulas; these make them bit-level)
 *   - round(x/s) is round-half-to-even of the exact product x * inv_s, inv_s = fl32(1/s).
 *   - the straight-through clamp indicator is taken on the rounded value, bounds inclusive.
 *   - dequantisation is one fp32 multiply then one round-to-nearest-even to the 16-bit type.
 */
#ifndef SASQ_H
#define SASQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SASQ_OK = 0,
    SASQ_ERR_NULL = 1,         /* a required pointer is NULL                               */
    SASQ_ERR_SHAPE = 2,        /* a size is <= 0, too large, or violates a stated multiple */
    SASQ_ERR_ALIGN = 3,        /* a base pointer is not 16-byte aligned                    */
    SASQ_ERR_UNSUPPORTED = 4,  /* unknown enum value or bits outside [2, 8]                */
    SASQ_ERR_WORKSPACE = 5,    /* workspace NULL or smaller than the matching query        */
    SASQ_ERR_LAUNCH = 6        /* the HIP runtime reported an error at launch              */
} sasq_status;

typedef enum { SASQ_F16 = 0, SASQ_BF16 = 1 } sasq_dtype;            /* activation / output type */
typedef enum {                       /* frozen weight storage                                    */
    SASQ_W_INT8 = 0,                 /* [N, K] int8, row-major                                   */
    SASQ_W_INT4_PACKED = 1,          /* [N, K/2] bytes, row-major, two codes per byte            */
    SASQ_W_INT8_BLOCKED = 2,         /* output of sasq_pack_weight from SASQ_W_INT8              */
    SASQ_W_INT4_BLOCKED = 3          /* output of sasq_pack_weight from SASQ_W_INT4_PACKED       */
} sasq_wfmt;

#define SASQ_MAX_BATCH 8                 /* tensors / projections per batched call                  */

/* Human-readable name of a status code (static storage, host pointer). */
const char* sasq_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int sasq_version(void);

/*
 * Test and tuning aid, not part of the method: force one of the library's kernel variants instead
 * of the choice the library makes from the shapes.  Every variant of a call computes the same
 * results bit for bit; the parity tests use this to cover each of them, the benchmark to compare
 * them.  The setting is process-wide and not thread-safe; value 0 restores the library's choice.
 * Unknown knob or value: SASQ_ERR_UNSUPPORTED.  The library reads no environment variables.
 */
typedef enum {
    SASQ_TUNE_LINEAR_PATH = 0,   /* 1: separate activation-quantize pass, 2: quantize on load          */
    SASQ_TUNE_LINEAR_TILE = 1,   /* 1: 256x256, 2: 128x256, 3: 128x128 workgroup tiles                  */
    SASQ_TUNE_LINEAR_MFMA = 2,   /* GEMMs: 1: the kernels on 32x32 MFMA tiles, 2: on 16x16 tiles (where they exist) */
    SASQ_TUNE_FQ_SHARE = 3,      /* 1..3: forward operators per group sharing one read of x, any size   */
    SASQ_TUNE_BWD_TILE = 4,      /* backward GEMM: 1: 256x256, 2: 128x128 tiles                         */
    SASQ_TUNE_COUNT = 5
} sasq_tune_knob;
int sasq_set_tuning(int knob, int value);

/*
 * Prepare a workspace for use by the calls below (zero-fills its control words, the first
 * 1024 bytes or the whole workspace if smaller, on `stream`).  Call once per workspace
 * allocation, before the first call that uses it.  Minimum size 256 bytes.
 */
int sasq_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/*
 * Fake quantization, forward (the operator Sec. 4.2 inserts before each linear; Sec. 3, Eq. 1;
 * dequantisation X' = S_x * X_int, Sec. 4.3, Eq. 5):
 *     q = clamp(round(x / s), -2^(bits-1), 2^(bits-1) - 1),   y = s * q.
 *   x      [rows, cols] device, 16-bit `dt`, read only
 *   s      device, one fp32: the per-tensor activation quantization factor
 *   y      [rows, cols] device, 16-bit `dt`, written (may alias x)
 *   codes  [rows, cols] device int8 or NULL: the integer codes q (for inspection and tests)
 *   bits   2..8
 */
int sasq_fakequant_fwd(const void* x, const float* s, void* y, int8_t* codes,
                       int64_t rows, int64_t cols, int bits, sasq_dtype dt, void* stream);

/* Bytes of workspace sasq_fakequant_bwd needs for this shape (pure function, host only). */
size_t sasq_fakequant_bwd_workspace(int64_t rows, int64_t cols);

/*
 * Fake quantization, backward with the straight-through estimator (Sec. 4.2, Eq. 4: the
 * gradient of round is 1, the gradient of clamp is 1 inside the range and 0 outside), and the
 * gradient of the scale, the only trained parameter (Sec. 4.2), by the chain rule:
 *     m  = 1 if -2^(bits-1) <= round(x/s) <= 2^(bits-1)-1 else 0
 *     dx = dy * m
 *     ds = sum over all elements of dy * (q - m * x/s)         (overwritten, not accumulated)
 *   x, dy  [rows, cols] device, 16-bit `dt`, read only
 *   s      device fp32 scalar
 *   dx     [rows, cols] device, 16-bit `dt`, written (may alias dy), or NULL to skip it
 *   ds     device fp32 scalar, written.  The reduction order is fixed: repeated calls with the
 *          same inputs give bit-identical results.
 *   workspace  >= sasq_fakequant_bwd_workspace(rows, cols) bytes, initialised once
 */
int sasq_fakequant_bwd(const void* x, const void* dy, const float* s, void* dx, float* ds,
                       int64_t rows, int64_t cols, int bits, sasq_dtype dt,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * sasq_fakequant_bwd for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs,
 * outputs, arithmetic and reduction order as sasq_fakequant_bwd (results are bit-identical); the
 * ticket word and the 256 fp64 block partials (3 KB) live in a device array that is part of the
 * library image instead of a caller workspace.  The call allocates nothing and frees nothing.
 *   - Each GPU holds one copy of that array for the life of the process; every call on a GPU uses
 *     it, so two calls that can overlap in time on one GPU (different streams) race: serialise them.
 *   - rows * cols above SASQ_FAKEQUANT_BWD_STATIC_MAX_ELEMENTS is rejected with SASQ_ERR_SHAPE.
 *   - The first call on a device looks the array's address up (no allocation); make that call
 *     outside graph capture.  A failed lookup returns SASQ_ERR_WORKSPACE.
 *   - Two kernels are enqueued: a one-thread clear of the ticket word, then the backward kernel.
 */
#define SASQ_FAKEQUANT_BWD_STATIC_MAX_ELEMENTS (INT64_C(1) << 40)
int sasq_fakequant_bwd_static(const void* x, const void* dy, const float* s, void* dx, float* ds,
                              int64_t rows, int64_t cols, int bits, sasq_dtype dt, void* stream);

/*
 * Per-channel variants of the fake-quant operator: one learned factor per activation channel
 * (column), the granularity of the paper's main experiments (Sec. 4; Sec. 5.1 "Implementation";
 * Sec. 2, Fig. 2(b)).  Same element arithmetic as above with s = s[k] for column k;
 *     ds[k] = sum over rows m of dy[m,k] * (q[m,k] - m[m,k] * x[m,k]/s[k])   (overwritten).
 *   s, ds   [cols] device fp32
 *   cols    at most 130560; the 128-bit path needs cols % 8 == 0, other widths take a slow
 *           one-thread-per-column kernel (and then need no workspace)
 * The per-channel backward uses one ticket per 512-column chunk of its workspace header; the
 * same workspace must not be shared with an overlapping call of any other entry point.
 */
int sasq_fakequant_fwd_pc(const void* x, const float* s, void* y, int8_t* codes,
                          int64_t rows, int64_t cols, int bits, sasq_dtype dt, void* stream);
size_t sasq_fakequant_bwd_pc_workspace(int64_t rows, int64_t cols);
int sasq_fakequant_bwd_pc(const void* x, const void* dy, const float* s, void* dx, float* ds,
                          int64_t rows, int64_t cols, int bits, sasq_dtype dt,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * The fake-quant operators of several tensors in one launch (a decoder layer has seven, one in
 * front of each linear, Sec. 4.2; at LLaMA-2-7B sizes a separate launch per tensor spends a fifth
 * of its time ramping up and draining).  Element arithmetic, outputs and error rules are those of
 * sasq_fakequant_fwd / sasq_fakequant_bwd applied to each item; ds of an item is reduced in a
 * fixed order that depends on the batch's composition only (deterministic from run to run; it may
 * differ from the single-tensor call's ds in the last bits).
 *   items   HOST array of `count` descriptors (1 <= count <= SASQ_MAX_BATCH), read before the call
 *           returns; the pointers inside are device pointers with the meaning of the single calls:
 *           x, s always; out = y (forward, required) or dx (backward, may be NULL); dy and ds
 *           backward only.  Items must not overlap each other's outputs.
 *   workspace (backward)  >= sasq_fakequant_bwd_batch_workspace(count) bytes, initialised once
 *           with sasq_workspace_init; not shared with an overlapping call.
 * Forward items that name the same x (same pointer, same rows * cols; the operators in front of
 * q/k/v or of gate/up read one activation tensor, each with its own factor) may be run together, up
 * to three at a time, x being read from memory once for the group (large tensors only).  Outputs
 * are unchanged.
 */
typedef struct {
    const void* x;      /* [rows, cols] device, 16-bit `dt`                      */
    const void* dy;     /* backward: [rows, cols] device, 16-bit `dt`            */
    const float* s;     /* device fp32 scalar                                     */
    void* out;          /* forward: y; backward: dx or NULL                       */
    float* ds;          /* backward: device fp32 scalar, overwritten              */
    int64_t rows, cols;
} sasq_fq_item;
int sasq_fakequant_fwd_batch(const sasq_fq_item* items, int count, int bits, sasq_dtype dt, void* stream);
size_t sasq_fakequant_bwd_batch_workspace(int count);
int sasq_fakequant_bwd_batch(const sasq_fq_item* items, int count, int bits, sasq_dtype dt,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same for per-channel factors (one factor per activation column, Sec. 4; Fig. 2(b)): each
 * item is a sasq_fakequant_fwd_pc / sasq_fakequant_bwd_pc call, `s` and `ds` pointing at `cols`
 * floats.  Outputs are bit-identical to the single-tensor calls (the column reduction of an item
 * does not depend on the batch).  Every item needs cols % 8 == 0 (SASQ_ERR_SHAPE otherwise: such
 * tensors take the single-tensor call), and the items of one backward call at most 256 column
 * blocks of 512 columns in all (SASQ_ERR_SHAPE; the workspace query then returns 0).
 *   workspace (backward)  >= sasq_fakequant_bwd_pc_batch_workspace(items, count) bytes, initialised
 *           once with sasq_workspace_init.
 */
int sasq_fakequant_fwd_pc_batch(const sasq_fq_item* items, int count, int bits, sasq_dtype dt, void* stream);
size_t sasq_fakequant_bwd_pc_batch_workspace(const sasq_fq_item* items, int count);
int sasq_fakequant_bwd_pc_batch(const sasq_fq_item* items, int count, int bits, sasq_dtype dt,
                                void* workspace, size_t workspace_bytes, void* stream);

/* SGD step of sasq_scale_sgd on a vector of n scales (the scales of one layer in one launch). */
int sasq_scale_sgd_vec(float* s, const float* ds, int64_t n, float lr, void* stream);

/*
 * One plain SGD step on the scale (the optimiser state of SASQ is the scale alone, Sec. 4.2;
 * the paper's own runs use AdamW, Sec. 5.1):  *s = fl32(*s - fl32(lr * *ds)).
 */
int sasq_scale_sgd(float* s, const float* ds, float lr, void* stream);

/*
 * One AdamW step (decoupled weight decay) on a vector of n scales, the optimiser of the paper's
 * runs (Sec. 5.1: AdamW, learning rate 2e-4; the scales are the only parameters, Sec. 4.2):
 *     p <- p - lr*wd*p;  m <- b1*m + (1-b1)*g;  v <- b2*v + (1-b2)*g^2;
 *     p <- p - lr * (m/(1-b1^step)) / (sqrt(v/(1-b2^step)) + eps)
 *   s, ds, m, v  [n] device fp32 (m, v: first and second moment state, zero before step 1)
 *   step         1-based step count.  Hyper-parameters are doubles (1 - beta is formed in double);
 *                the update itself is fp32 arithmetic and agrees with an fp64 evaluation to ~1e-6 relative.
 */
int sasq_scale_adamw(float* s, const float* ds, float* m, float* v, int64_t n, int64_t step,
                     double lr, double beta1, double beta2, double eps, double weight_decay, void* stream);

/* Bytes of workspace sasq_static_linear needs (pure function, host only; may be 0). */
size_t sasq_static_linear_workspace(int64_t M, int64_t N, int64_t K, sasq_wfmt wf);

/*
 * Static-inference quantized linear (Sec. 3, Eq. 2: Y = S_x * (X_int . W_int) * S_w, integer
 * product first, inverse quantization after; bias not quantized).  The activation scale is a
 * fixed input: nothing is reduced over X at run time (static quantization, Sec. 3; Sec. 4.5).
 *     xq[m,k]  = clamp(round(X[m,k] / s), -2^(a_bits-1), 2^(a_bits-1) - 1)
 *     acc[m,n] = sum_k xq[m,k] * Wq[n,k]                      (exact, int32)
 *     Y[m,n]   = fl32(fl32(acc[m,n]) * fl32(s * s_w[n])) (+ bias[n])  -> 16-bit `dt`
 *   x        [M, K] device 16-bit `dt`
 *   s        device fp32 scalar
 *   wq       [N, K] device int8 (SASQ_W_INT8), or [N, K/2] bytes (SASQ_W_INT4_PACKED): element k
 *            even in the low nibble, k odd in the high nibble, two's complement, range [-8, 7];
 *            or the sasq_packed_weight_bytes(N, K, wf) bytes sasq_pack_weight made of either
 *            (SASQ_W_INT8_BLOCKED, SASQ_W_INT4_BLOCKED: same codes, same results bit for bit,
 *            arranged so that the GEMM reads them in whole cache lines; the fast path for
 *            frozen weights; K must be a multiple of 64, else SASQ_ERR_SHAPE)
 *   s_w      [N] device fp32, one factor per output channel
 *   bias     [N] device fp32 or NULL
 *   y        [M, N] device 16-bit `dt`, written
 *   acc_out  [M, N] device int32 or NULL; xq_out [M, K] device int8 or NULL (inspection/tests;
 *            requesting either selects a slower code path)
 *   K        multiple of 2 for int4.  Any M, N, K > 0 is accepted; the MFMA path is taken when
 *            K is a multiple of 64, other shapes use a scalar kernel.
 *   M*K, N*K, M*N must each be < 2^40; |acc| cannot overflow for K <= 131071.
 *   workspace  >= sasq_static_linear_workspace(M, N, K, wf) bytes (NULL allowed when that is 0);
 *              holds the int8 activation codes in a library-internal blocked order between the
 *              quantize pass and the GEMM; contents after the call are unspecified
 */
int sasq_static_linear(const void* x, const float* s, const void* wq, const float* s_w,
                       const float* bias, void* y, int32_t* acc_out, int8_t* xq_out,
                       int64_t M, int64_t N, int64_t K, int a_bits, sasq_wfmt wf, sasq_dtype dt,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * The static linears of several projections (one decoder layer) in two launches: one activation
 * pre-pass and one GEMM over the tiles of all projections, longest K first, so that the layer pays
 * one launch ramp and one drain and the partly filled last round of a projection is filled by the
 * next one's tiles.  Arithmetic and results of each item are exactly those of sasq_static_linear.
 *   items   HOST array of `count` descriptors (1 <= count <= SASQ_MAX_BATCH), read before the call
 *           returns; pointers inside are device pointers as in sasq_static_linear (bias may be NULL).
 *           Every K must be a multiple of 64 (SASQ_ERR_SHAPE otherwise: use the single call).
 *   a_bits, wf, dt   shared by all items.  No inspection outputs.
 *   workspace >= sasq_static_linear_batch_workspace(items, count, wf) bytes.
 */
typedef struct {
    const void* x;        /* [M, K] device, 16-bit `dt`                 */
    const float* s;       /* device fp32 scalar                          */
    const void* wq;       /* weights in format `wf`                      */
    const float* s_w;     /* [N] device fp32                             */
    const float* bias;    /* [N] device fp32 or NULL                     */
    void* y;              /* [M, N] device, 16-bit `dt`, written         */
    int64_t M, N, K;
} sasq_linear_item;
size_t sasq_static_linear_batch_workspace(const sasq_linear_item* items, int count, sasq_wfmt wf);
int sasq_static_linear_batch(const sasq_linear_item* items, int count, int a_bits, sasq_wfmt wf,
                             sasq_dtype dt, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Static-inference quantized linear with one activation factor per group of `group` consecutive
 * input channels (Sec. 3, Eq. 3: Y = sum_i (S_x,i * S_w) * (X_int,i . W_int), the block-wise form
 * the paper gives for activations quantized per channel; Sec. 4 trains per-channel factors):
 *     xq[m,k]    = clamp(round(X[m,k] / s_g[k / group]), -2^(a_bits-1), 2^(a_bits-1) - 1)
 *     acc_i[m,n] = sum over the k of group i of xq[m,k] * Wq[n,k]          (exact, int32)
 *     f[m,n]     = fma(fl32(acc_i[m,n]), s_g[i], f[m,n]) for i = 0 .. K/group - 1, from f = 0
 *     Y[m,n]     = fl32(f[m,n] * s_w[n]) (+ bias[n])  -> 16-bit `dt`
 * (the paper fixes no rounding order for Eq. 3; this one is what the kernels and the test oracle
 * share.)  group = 1 is per-channel in the strict sense, group = K a per-tensor factor.
 *   s_g      [K / group] device fp32
 *   f_out    [M, N] device fp32 or NULL: f, for inspection and tests (slower path); xq_out as in
 *            sasq_static_linear
 *   group    divides K.  The MFMA path is taken when K and group are multiples of 64 (then all
 *            four weight formats are accepted), and for group = 32 with K a multiple of 64 and
 *            any format but row-major int4 (each 64-channel K tile is then multiplied twice, one
 *            half of the channels at a time); other shapes run a scalar kernel and accept the
 *            row-major weight formats only (SASQ_ERR_SHAPE for the pre-arranged ones).
 *   every other argument, the workspace size and the limits are those of sasq_static_linear.
 */
int sasq_static_linear_grouped(const void* x, const float* s_g, const void* wq, const float* s_w,
                               const float* bias, void* y, float* f_out, int8_t* xq_out,
                               int64_t M, int64_t N, int64_t K, int64_t group, int a_bits,
                               sasq_wfmt wf, sasq_dtype dt, void* workspace, size_t workspace_bytes,
                               void* stream);

/*
 * Dynamic per-token quantized linear: the baseline whose online step the static factors remove
 * (Sec. 3: dynamic quantization computes the factors during inference, per-token = one factor per
 * row of X; Sec. 4.5 compares against it).  For every row m:
 *     s_m      = fl32(max_k |X[m,k]| / (2^(a_bits-1) - 1))      (1 if the row is all zero)
 *     xq[m,k]  = clamp(round(X[m,k] / s_m), -2^(a_bits-1), 2^(a_bits-1) - 1)
 *     acc[m,n] = sum_k xq[m,k] * Wq[n,k]                        (exact, int32)
 *     Y[m,n]   = fl32(fl32(acc[m,n]) * fl32(s_m * s_w[n])) (+ bias[n])  -> 16-bit `dt`
 *   x must be finite.  s_row_out [M] device fp32 or NULL: the factors (inspection, tests, or use as
 *   an absmax calibration pass).  acc_out, xq_out, wq, s_w, bias, y, shapes, weight formats
 *   and limits as in sasq_static_linear.
 *   workspace >= sasq_dynamic_linear_workspace(M, N, K, wf) bytes.
 */
size_t sasq_dynamic_linear_workspace(int64_t M, int64_t N, int64_t K, sasq_wfmt wf);
int sasq_dynamic_linear(const void* x, const void* wq, const float* s_w, const float* bias, void* y,
                        int32_t* acc_out, int8_t* xq_out, float* s_row_out,
                        int64_t M, int64_t N, int64_t K, int a_bits, sasq_wfmt wf, sasq_dtype dt,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Quantize frozen weights, symmetric, one factor per output channel (Sec. 3, Eq. 1 applied to
 * each row of W[N,K]; Sec. 5.1 fixes the weight granularity to per output channel):
 *     s_w[n]  = fl32(max_k |W[n,k]| / Qp)     (1 if the row is all zero),  Qp = 127 or 7
 *     Wq[n,k] = clamp(round(W[n,k] / s_w[n]), -Qp-1, Qp)     (same rounding rule as activations)
 *   w    [N, K] device fp32;  wq: [N, K] int8 or [N, K/2] packed int4 (K even);  s_w [N] fp32
 */
int sasq_quantize_weight(const float* w, void* wq, float* s_w, int64_t N, int64_t K,
                         sasq_wfmt wf, void* stream);

/*
 * Re-arrange quantized frozen weights for the GEMM (a set-up step, once per weight matrix; the
 * weights of static inference never change, Sec. 3).  A pure permutation of the codes:
 *   SASQ_W_INT8 -> SASQ_W_INT8_BLOCKED: 1 KB blocks of 16 rows x 64 K-bytes, block (n/16, k/64) at
 *     ((n/16) * K/64 + k/64) * 1024; inside, the 16-byte chunk c of row r at
 *     16 * (4r + (c ^ ((r >> 1) & 3) ^ ((r >> 3) & 1))).
 *   SASQ_W_INT4_PACKED -> SASQ_W_INT4_BLOCKED: 1 KB blocks of 32 rows x 64 k, block (n/32, k/64) at
 *     ((n/32) * K/64 + k/64) * 1024; the 16 codes k = 64*(k/64) + 32*kk + 16*g + (0..15) of row r
 *     are the 8 bytes at 512*kk + 256*g + 8*r: byte b of the first four holds code b (low nibble)
 *     and code 4+b (high nibble), byte b of the last four codes 8+b and 12+b.
 * Rows past N in the last block are zero.
 *   wq       device, row-major codes in format wf_src (SASQ_W_INT8 or SASQ_W_INT4_PACKED)
 *   packed   device, sasq_packed_weight_bytes(N, K, blocked format) bytes, written; not wq
 *   K        multiple of 64 (SASQ_ERR_SHAPE otherwise: use the row-major format for such shapes)
 * sasq_packed_weight_bytes is a pure host function; it returns 0 for shapes or formats that have
 * no blocked form.
 */
size_t sasq_packed_weight_bytes(int64_t N, int64_t K, sasq_wfmt wf);
int sasq_pack_weight(const void* wq, void* packed, int64_t N, int64_t K, sasq_wfmt wf_src, void* stream);

/*
 * Backward of the frozen quantized linear with respect to its input: the step that hands each
 * fake-quant operator its upstream gradient during scale training (Sec. 4.2; the weight is
 * Eq. 2's W_int * S_w, frozen):
 *     Wq[n,k] = round16(fl32(fl32(W_int[n,k]) * s_w[n]))        (prepared once)
 *     dX[m,k] = round16(sum_n dY[m,n] * Wq[n,k])                 (16-bit MFMA, fp32 accumulation)
 * The sum's rounding order is the matrix unit's: dX agrees with the exactly rounded result within
 * the fp32 accumulation bound N * 2^-24 * sum_n |dY[m,n] * Wq[n,k]| plus one 16-bit rounding.
 *
 * sasq_prepare_bwd_weight writes Wq transposed and cut into the GEMM's operand blocks:
 *   B[k][n] = Wq[n][k]; 1 KB blocks of 16 rows (k) x 32 columns (n), block (k/16, n/32) at
 *   ((k/16) * ceil(N/32) + n/32) * 1024; inside, the 16-byte chunk c (8 columns) of row r at
 *   16 * (4r + (c ^ ((r >> 1) & 3) ^ ((r >> 3) & 1))).  Rows past K and columns past N are zero.
 *   wq       device, row-major codes [N,K], SASQ_W_INT8 or SASQ_W_INT4_PACKED
 *   s_w      device, N floats
 *   wt       device, sasq_bwd_weight_bytes(N, K) bytes, 16-byte aligned, written
 *   N        any; the MFMA kernel runs when N is a multiple of 32, a scalar kernel otherwise
 * sasq_linear_bwd_input:
 *   dy       device, [M,N] row-major 16-bit, 16-byte aligned, read only
 *   wt       device, as prepared for the same N, K and dt
 *   dx       device, [M,K] row-major 16-bit, 16-byte aligned, written; must not alias dy
 *   acc_out  device, optional (NULL to skip): [M,K] floats, the fp32 sums before the 16-bit rounding
 * sasq_bwd_weight_bytes is a pure host function.
 */
size_t sasq_bwd_weight_bytes(int64_t N, int64_t K);
int sasq_prepare_bwd_weight(const void* wq, const float* s_w, void* wt, int64_t N, int64_t K,
                            sasq_wfmt wf, sasq_dtype dt, void* stream);
int sasq_linear_bwd_input(const void* dy, const void* wt, void* dx, float* acc_out,
                          int64_t M, int64_t N, int64_t K, sasq_dtype dt, void* stream);

/* Bytes of workspace sasq_absmax_scale needs (pure function, host only). */
size_t sasq_absmax_scale_workspace(int64_t rows, int64_t cols);

/*
 * Initial (post-training) scale of an activation tensor (Sec. 3, Eq. 1, right half; Sec. 4.1):
 *     *s = fl32(max|x| / (2^(bits-1) - 1)).
 * This is the dynamic-quantization reduction that static inference avoids; it is used once,
 * to initialise s before training.
 */
int sasq_absmax_scale(const void* x, float* s, int64_t rows, int64_t cols, int bits,
                      sasq_dtype dt, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SASQ_H */
