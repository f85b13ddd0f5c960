/*
 * txops.h -- C ABI of the MI355X (gfx950) ATen-semantics operator library.
 *
 * The library executes the operator classes that the paper's agent generates
 * kernels for (Section 3.3: the ATen operator set exercised by OpInfo, dtypes
 * bf16 / fp16 / fp32 / int32 / int64, here plus bool; Table 1 categories
 * Elementwise, Reduction, Indexing & Selection, and softmax from Deep
 * Learning).  A call must return what the ATen CPU operator returns on the
 * same strided, typed operands (Section 3.2, the test runner's criterion);
 * the paper delegates the per-operator semantics to the PyTorch operator
 * documentation, and the comments below restate the parts that matter.
 *
 * General conventions
 *   - Every tensor argument is a host pointer to a tx_tensor descriptor whose
 *     `data` member is a DEVICE pointer to element [0,...,0] (storage offset
 *     applied).  Sizes are >= 0, strides are in ELEMENTS, 0 strides are
 *     allowed on inputs (broadcast views), negative strides are not allowed.
 *     ndim == 0 describes a one-element tensor.
 *   - Ownership: the caller owns every buffer, workspace included.  The
 *     library allocates no device memory and keeps no pointer after return.
 *   - `stream` is a hipStream_t (pass NULL for the default stream).  All work
 *     is enqueued on it and the call returns without synchronising; buffers
 *     and workspace must stay alive until the stream has passed the call.
 *   - Errors: every semantic check happens on the host before any launch.  A
 *     negative tx_status is returned, nothing is written, and
 *     tx_last_error() holds a thread-local detail string.
 *   - numel(out) == 0 returns TX_OK without launching.
 *   - `out` must have exactly the inferred shape.  Its dtype must be the
 *     inferred result dtype, except where a function says otherwise: tx_unary,
 *     tx_add / tx_sub / tx_binary and tx_clamp accept any out dtype the result
 *     dtype can be cast to (ATen's `out=` rule: no floating result into an
 *     integer or bool tensor, no integer result into a bool tensor); the
 *     result is formed and rounded in the result dtype first, then converted
 *     (integers narrow by wrapping and reach a half dtype through fp32).
 *     `out` may have any non-overlapping strides.  It may alias an input
 *     exactly (same pointer, sizes and strides).  Together these give the
 *     in-place variants: a.add_(b) is tx_add(out = a, a, b), legal whenever
 *     the promoted dtype can be cast to a's.  Any other overlap between `out`
 *     and an input, and any self-overlap inside `out`, is TX_ERR_OVERLAP.
 *   - Type promotion (binary ops, where): categories bool < integer <
 *     floating.  Operands with ndim >= 1 are promoted among themselves and
 *     0-dim operands among themselves (wider wins inside a category, fp16
 *     with bf16 gives fp32, a higher category wins unchanged); the 0-dim group
 *     decides only when its category is strictly higher.  Operands are
 *     converted to the common dtype first, then the operator is applied;
 *     fp16 / bf16 arithmetic is carried out in fp32 and rounded once
 *     (nearest-even) on store.
 */
#ifndef TXOPS_H
#define TXOPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types; bool is one byte holding 0 or 1 */
enum { TX_BOOL = 0, TX_I32 = 1, TX_I64 = 2, TX_F16 = 3, TX_BF16 = 4, TX_F32 = 5 };

#define TX_MAX_DIMS 8

typedef struct {
  void* data;                   /* device pointer */
  int32_t dtype;                /* TX_* element type */
  int32_t ndim;                 /* 0..TX_MAX_DIMS */
  int64_t sizes[TX_MAX_DIMS];
  int64_t strides[TX_MAX_DIMS]; /* in elements */
} tx_tensor;

typedef int32_t tx_status;
enum {
  TX_OK = 0,
  TX_ERR_NULL = -1,            /* null descriptor, or null data with numel > 0 */
  TX_ERR_NDIM = -2,            /* ndim outside 0..TX_MAX_DIMS */
  TX_ERR_DTYPE = -3,           /* dtype not valid for the op, or out dtype != inferred */
  TX_ERR_SHAPE = -4,           /* not broadcastable, wrong out shape, index shape rules, negative size/stride */
  TX_ERR_DIM = -5,             /* dim out of range or repeated; several dims for prod / argmax */
  TX_ERR_OVERLAP = -6,         /* out overlaps itself or partially overlaps an input */
  TX_ERR_EMPTY_REDUCTION = -7, /* amax / amin / argmax / argmin over an empty reduced extent */
  TX_ERR_SCALAR = -8,          /* non-integral alpha with an integer / bool result */
  TX_ERR_WORKSPACE = -9,       /* workspace missing or smaller than tx_*_workspace_bytes() */
  TX_ERR_INDEX = -10,          /* an index value out of range: only with index validation on (tx_set_index_validation) */
  TX_ERR_LAUNCH = -11,         /* HIP reported an error at launch; see tx_last_error() */
  TX_ERR_UNSUPPORTED = -12     /* valid request that this build has no kernel for */
};

/* operator codes */
enum { TX_NEG = 0, TX_ABS, TX_EXP, TX_LOG, TX_SQRT, TX_SIGMOID, TX_TANH, TX_GELU_ERF, TX_LOG1P, TX_EXPM1, TX_LOGSIGMOID,
       TX_LOGICAL_NOT, TX_SIN, TX_COS, TX_EXP2, TX_LOG2, TX_LOG10, TX_RSQRT, TX_RECIPROCAL, TX_SILU, TX_SQUARE, TX_SIGN,
       TX_FLOOR, TX_CEIL, TX_TRUNC, TX_ROUND, TX_ISNAN, TX_ISINF, TX_ISFINITE, TX_BITWISE_NOT, TX_TAN, TX_ASIN, TX_ACOS,
       TX_ATAN, TX_SINH, TX_COSH, TX_ASINH, TX_ACOSH, TX_ATANH, TX_ERF, TX_ERFC, TX_RELU, TX_FRAC, TX_SIGNBIT,
       TX_HARDSWISH, TX_HARDSIGMOID, TX_MISH };
enum { TX_ADD = 0, TX_MUL, TX_DIV, TX_MAXIMUM, TX_EQ, TX_SUB, TX_MINIMUM, TX_NE, TX_LT, TX_LE, TX_GT, TX_GE,
       TX_LOGICAL_AND, TX_LOGICAL_OR, TX_LOGICAL_XOR, TX_POW, TX_BITWISE_AND, TX_BITWISE_OR, TX_BITWISE_XOR, TX_ATAN2,
       TX_FMOD, TX_REMAINDER, TX_HYPOT, TX_COPYSIGN, TX_LOGADDEXP, TX_LOGADDEXP2, TX_XLOGY, TX_HEAVISIDE, TX_FMAX,
       TX_FMIN, TX_NEXTAFTER, TX_GCD, TX_LCM, TX_SHIFT_LEFT, TX_SHIFT_RIGHT, TX_FLOOR_DIVIDE, TX_TRUNC_DIVIDE };
enum { TX_SUM = 0, TX_MEAN, TX_AMAX, TX_ARGMAX, TX_PROD, TX_VAR, TX_AMIN, TX_ARGMIN, TX_STD, TX_ANY, TX_ALL,
       TX_LOGSUMEXP, TX_NANSUM, TX_NANMEAN, TX_COUNT_NONZERO, TX_NORM };

/* ------------------------------------------------------------------ elementwise
 * (Table 1 "Elementwise"; the flat masked kernels of Appendix B are the paper's
 * form of this class, the `outer` listing its broadcasting form.)
 */

/* out[i] = f(a[i]); out has a's shape.
 *   NEG, ABS : result dtype = a's; bool is TX_ERR_DTYPE; integers wrap; floats
 *              flip / clear the sign bit exactly.
 *   EXP LOG SQRT SIGMOID TANH LOG1P EXPM1 : float a keeps its dtype; bool /
 *              integer a is converted to fp32 and the result is fp32.  fp32
 *              results are within 2 ulp of the correctly rounded value.
 *   GELU_ERF : x * Phi(x); float dtypes only.
 *   LOGSIGMOID : log(1 / (1 + exp(-x))) (Appendix D's worked example), float
 *              dtypes only, evaluated as min(x, 0) - log1p(exp(-|x|)).
 *   LOGICAL_NOT : x == 0 for any dtype (a NaN is not zero), bool result.
 *   SIN COS EXP2 LOG2 LOG10 RSQRT RECIPROCAL : like EXP (RSQRT = 1 / sqrt(x)).
 *   SILU : x / (1 + exp(-x)); float dtypes only.
 *   SQUARE : x * x; integers wrap; a bool gives the int64 0 / 1.
 *   SIGN : -1, 0 or 1 in a's dtype; 0 for a NaN and for either zero; a bool is
 *              returned unchanged.
 *   FLOOR CEIL TRUNC ROUND : floats (ROUND: halves to even; the sign of zero is
 *              kept); integers are returned unchanged; bool is TX_ERR_DTYPE.
 *   ISNAN ISINF ISFINITE : any dtype, bool result (integers are finite).
 *   BITWISE_NOT : ~x for integers, logical not for bool; floats are TX_ERR_DTYPE.
 *   TAN ASIN ACOS ATAN SINH COSH ASINH ACOSH ATANH ERF ERFC : like EXP.
 *   RELU : x < 0 ? 0 : x (a NaN and -0.0 stay); integers too; bool is
 *              TX_ERR_DTYPE.
 *   FRAC : x - trunc(x).  HARDSIGMOID : min(max(x + 3, 0), 6) / 6.  HARDSWISH :
 *              x times that.  MISH : x * tanh(log1p(exp(x))).  Float dtypes
 *              only; fp32 results within 2 ulp.
 *   SIGNBIT : the sign bit of a float (-0.0 and negative NaNs included), x < 0
 *              for an integer, false for a bool; bool result. */
tx_status tx_unary(int op, const tx_tensor* out, const tx_tensor* a, void* stream);

/* Unary operators with scalar parameters (Table 1 "Deep Learning" activations and
 * their relatives): out[i] = f(a[i]; p0, p1, p2), out has a's shape and the
 * result dtype.  The parameters are binary64 values; fp32 results are within
 * 2 ulp of the binary64 evaluation.
 *   LEAKY_RELU(p0 = slope)   x > 0 ? x : x * slope
 *   ELU(p0 = alpha)          x > 0 ? x : alpha * expm1(x)
 *   CELU(p0 = alpha)         x > 0 ? x : alpha * expm1(x / alpha); alpha = 0 is
 *                            TX_ERR_SCALAR
 *   SELU                     scale * ELU(alpha) with the two published constants
 *   SOFTPLUS(p0 = beta, p1 = threshold)  x * beta > threshold ? x :
 *                            log1p(exp(x * beta)) / beta
 *   HARDSHRINK(p0 = lambda)  -lambda <= x <= lambda ? 0 : x
 *   SOFTSHRINK(p0 = lambda)  x > lambda ? x - lambda : x < -lambda ? x + lambda :
 *                            x * 0; a negative lambda is TX_ERR_SCALAR
 *       - floating dtypes only for these seven -
 *   THRESHOLD(p0 = threshold, p1 = value)  x <= threshold ? value : x; floats,
 *                            int32, int64 (parameters truncated to the integer
 *                            dtype); a NaN x stays
 *   LOGIT(p0 = eps, p1 != 0: eps given)  log(z / (1 - z)), z = x clamped to
 *                            [eps, 1 - eps] when eps is given; bool / integer a
 *                            computes and returns fp32
 *   NAN_TO_NUM(p0, p1, p2)   NaN, +inf, -inf replaced by the parameters rounded
 *                            to the dtype; bool / integer a is copied
 *   ROUND_DECIMALS(p0 = d)   d > 0: rint(x * 10^d) / 10^d; d < 0: rint(x / 10^-d)
 *                            * 10^-d; every step in fp32 (that arithmetic is the
 *                            operator's definition); d must be an integer with
 *                            |d| <= 38 (TX_ERR_SCALAR); floating dtypes only
 *   GELU_TANH                x (1 + tanh u) / 2, u = sqrt(2/pi)(x + 0.044715 x^3),
 *                            evaluated as x / (1 + exp(-2u)); floating dtypes only */
enum { TX_LEAKY_RELU = 0, TX_ELU, TX_CELU, TX_SELU, TX_SOFTPLUS, TX_THRESHOLD, TX_HARDSHRINK, TX_SOFTSHRINK, TX_LOGIT,
       TX_NAN_TO_NUM, TX_ROUND_DECIMALS, TX_GELU_TANH };
tx_status tx_unary_param(int op, const tx_tensor* out, const tx_tensor* a, double p0, double p1, double p2, void* stream);
int32_t tx_infer_unary_param_dtype(int op, int32_t in_dtype);

/* Ternary operators with broadcasting and type promotion.
 *   ADDCMUL  a + value * b * c; integer result: wrapping, value truncated; three
 *            bools are TX_ERR_DTYPE.
 *   ADDCDIV  a + value * b / c; the promoted dtype must be floating.
 *   LERP     a + w (b - a) for w < 1/2, b - (b - a)(1 - w) otherwise; w is the
 *            tensor c, or the scalar value when c is NULL; one floating dtype
 *            for every tensor.
 * value is given both ways (value_is_int selects value_i).  fp32 results are the
 * binary64 evaluation rounded once. */
enum { TX_ADDCMUL = 0, TX_ADDCDIV = 1, TX_LERP = 2 };
tx_status tx_ternary(int op, const tx_tensor* out, const tx_tensor* a, const tx_tensor* b, const tx_tensor* c, double value_f,
                     int64_t value_i, int value_is_int, void* stream);
int32_t tx_infer_ternary_dtype(int op, const tx_tensor* a, const tx_tensor* b, const tx_tensor* c);

/* add (Table 1 "Elementwise", the paper's largest category; the operator every
 * flat masked kernel of Appendix B is a variation of; accepted when its output
 * equals the ATen CPU operator's, Section 3.2).
 * out = a + alpha * b with broadcasting and type promotion.  alpha is given
 * both ways: alpha_is_int selects alpha_i, else alpha_f.  bool: a OR (alpha!=0
 * AND b).  Integer result: wrapping arithmetic, alpha must be integral
 * (TX_ERR_SCALAR otherwise).  Float result: alpha == 1 is one IEEE add;
 * alpha != 1 is one fused multiply-add fma(alpha, b, a) in fp32. */
tx_status tx_add(const tx_tensor* out, const tx_tensor* a, const tx_tensor* b, double alpha_f, int64_t alpha_i,
                 int alpha_is_int, void* stream);

/* out = a - alpha * b: tx_add's rules with the sign of the second term
 * reversed (float result: alpha == 1 is one IEEE subtraction, otherwise one
 * fma(-alpha, b, a) in fp32).  A bool operand is TX_ERR_DTYPE. */
tx_status tx_sub(const tx_tensor* out, const tx_tensor* a, const tx_tensor* b, double alpha_f, int64_t alpha_i,
                 int alpha_is_int, void* stream);

/* out = a (op) b with broadcasting and type promotion, op in MUL DIV MAXIMUM
 * MINIMUM EQ NE LT LE GT GE LOGICAL_AND LOGICAL_OR LOGICAL_XOR POW BITWISE_AND
 * BITWISE_OR BITWISE_XOR ATAN2 FMOD REMAINDER HYPOT COPYSIGN LOGADDEXP
 * LOGADDEXP2 XLOGY HEAVISIDE FMAX FMIN NEXTAFTER GCD LCM SHIFT_LEFT
 * SHIFT_RIGHT FLOOR_DIVIDE TRUNC_DIVIDE (TX_ADD and TX_SUB are accepted too,
 * with alpha = 1).
 *   MUL: bool AND, integers wrap.  DIV: true division, bool / integer pairs are
 *   computed and returned in fp32.  MAXIMUM / MINIMUM: NaN if either operand is
 *   NaN; on ties the first operand; bool OR / AND.
 *   EQ NE LT LE GT GE: compare in the common dtype, result dtype bool (IEEE:
 *   every ordered comparison with a NaN is false, NE is true).
 *   LOGICAL_AND / OR / XOR: (a != 0) op (b != 0) in the common dtype, result
 *   dtype bool; a NaN counts as non-zero.
 *   POW: a to the power b.  Floating common dtype: IEEE pow with the C Annex F
 *   special values (x^0 = 1 and 1^y = 1 even for NaN, negative base with a
 *   non-integer exponent = NaN), fp32 results within 2 ulp.  Integer common
 *   dtype: wrapping product; a negative exponent gives the truncated
 *   reciprocal (1 for base 1, +-1 for base -1 by parity, else 0).  Two bool
 *   operands are TX_ERR_DTYPE.
 *   BITWISE_AND / OR / XOR: on the integers of the common dtype (bool: the
 *   logical operation); a floating common dtype is TX_ERR_DTYPE.
 *   ATAN2: the angle of the point (b, a); bool / integer pairs are computed and
 *   returned in fp32; fp32 results within 2 ulp.
 *   FMOD: the remainder with the dividend's sign; REMAINDER: with the
 *   divisor's (fmod, plus the divisor when the signs differ and the value is
 *   not zero).  Exact for floats up to REMAINDER's one addition.  Two bools are
 *   TX_ERR_DTYPE.  An integer zero divisor is outside the contract: the
 *   device cannot report it and writes 0 there.
 *   HYPOT: sqrt(a^2 + b^2) without overflow, +inf when either is infinite.
 *   LOGADDEXP / LOGADDEXP2: log(e^a + e^b) and its base-2 form, equal
 *   infinities give themselves.  NEXTAFTER: the neighbour of a toward b in the
 *   common format.  These four need a floating common dtype.
 *   COPYSIGN: |a| with b's sign bit.  XLOGY: NaN if b is NaN, else 0 if
 *   a == 0, else a * log(b).  bool / integer pairs compute and return fp32.
 *   HEAVISIDE: 0 for a < 0 and for a NaN a, 1 for a > 0, b for a == 0; the
 *   two dtypes must be equal (TX_ERR_DTYPE otherwise).
 *   FMAX / FMIN: the larger / smaller; NaN only when both are NaN.
 *   GCD / LCM: of the magnitudes, wrapped to the dtype (gcd(0, 0) = lcm(0, x) =
 *   0).  SHIFT_LEFT / SHIFT_RIGHT: a << b and the arithmetic a >> b; a count
 *   below 0 or at least the width gives 0, or -1 for a negative a shifted
 *   right.  int32 / int64 only (a bool beside an integer promotes).
 *   FLOOR_DIVIDE / TRUNC_DIVIDE (Table 1, elementwise; ATen's div with a
 *   rounding mode): the quotient rounded toward -infinity / toward zero, in
 *   the common dtype (integers stay integers and wrap; two bools are
 *   TX_ERR_DTYPE; an integer zero divisor is outside the contract, 0 is
 *   written).  Floating operands are divided in binary32.  TRUNC truncates
 *   the quotient after rounding it to the common dtype (in bf16, 5.99 / 1 is
 *   6); FLOOR is rounded to the common dtype once at the end and starts from
 *   the exact fmod, (a - fmod(a, b)) / b, so a
 *   quotient just below an integer is not rounded up to it; zero results
 *   carry the quotient's sign and x / 0 is the IEEE quotient. */
tx_status tx_binary(int op, const tx_tensor* out, const tx_tensor* a, const tx_tensor* b, void* stream);

/* out = min(max(x, lo), hi) with scalar bounds; has_lo / has_hi say which are
 * present (neither: TX_ERR_SCALAR), each given both ways like alpha.  Result
 * dtype: x's, except integer x with a floating bound gives fp32; bool x is
 * TX_ERR_DTYPE.  x and the bounds are converted to the result dtype first (an
 * integer bound outside an int32 result's range is TX_ERR_SCALAR).  lo > hi
 * gives hi everywhere; a NaN in x stays; a NaN bound makes every output NaN. */
tx_status tx_clamp(const tx_tensor* out, const tx_tensor* x, int has_lo, double lo_f, int64_t lo_i, int lo_is_int,
                   int has_hi, double hi_f, int64_t hi_i, int hi_is_int, void* stream);

/* where (Table 1 "Elementwise": a three-operand operator whose operands have
 * three different roles; Section 3.2's criterion applied to the ATen operator
 * `where(cond, x, y)`).
 * out = cond ? x : y.  cond must be bool; result dtype = promotion of x and y;
 * the three operands broadcast together.  With no conversion the selected
 * element's bits are copied unchanged (NaN payloads survive). */
tx_status tx_where(const tx_tensor* out, const tx_tensor* cond, const tx_tensor* x, const tx_tensor* y, void* stream);

/* masked_fill (Table 1 "Indexing & Selection": selection by a boolean mask, the
 * case with a scalar payload; same acceptance criterion, Section 3.2).
 * out = mask ? value : self.  mask is bool and broadcasts with self; out has
 * the broadcast shape and self's dtype.  value is cast to self's dtype
 * (floating value into an integer dtype truncates toward zero). */
tx_status tx_masked_fill(const tx_tensor* out, const tx_tensor* self, const tx_tensor* mask, double value_f,
                         int64_t value_i, int value_is_int, void* stream);

/* ------------------------------------------------------------------ fused row / loss operators
 * (Table 1 "Deep Learning"; Appendix B.3 and B.1 print the paper's kernels
 * for these two operators.)
 */

/* layer_norm over the last norm_ndim dims of x (1 <= norm_ndim <= x.ndim, else
 * TX_ERR_DIM): per row of those dims, mean and biased variance, then
 *   out = (x - mean) / sqrt(var + eps) * weight + bias.
 * weight and bias are optional (NULL); each must have exactly the shape of the
 * normalised dims (TX_ERR_SHAPE) and x's dtype or fp32.  Floating dtypes only;
 * out has x's shape and dtype and may not alias an input (TX_ERR_OVERLAP).
 * Any strides; statistics are accumulated in fp32 (two passes over the row). */
tx_status tx_layer_norm(const tx_tensor* out, const tx_tensor* x, int32_t norm_ndim, const tx_tensor* weight,
                        const tx_tensor* bias, double eps, void* stream);

enum { TX_REDUCTION_NONE = 0, TX_REDUCTION_MEAN = 1, TX_REDUCTION_SUM = 2 };

/* loss = -weight * (target * max(ln input, -100) + (1 - target) * max(ln(1 - input), -100)).
 * input and target have the same shape and floating dtype; weight is optional
 * (NULL), floating, and broadcasts to input's shape.  input is meant to lie in
 * [0, 1]; this is not checked on the device (values outside give NaN).
 * reduction NONE: out has input's shape and dtype (it may alias an input
 * exactly); no workspace.  MEAN / SUM: out is 0-dim (mean of no elements: NaN),
 * accumulated in fp32 per lane and binary64 across lanes; needs a 16-byte
 * aligned device workspace of tx_binary_cross_entropy_workspace_bytes() bytes
 * (TX_ERR_WORKSPACE otherwise): partial sums, plus the losses themselves when
 * the operands cannot be read linearly (input and target not laid out alike,
 * or a weight that is neither laid out like input nor one value per element
 * of the last dim).  Other reduction codes are TX_ERR_SCALAR. */
tx_status tx_binary_cross_entropy(const tx_tensor* out, const tx_tensor* input, const tx_tensor* target,
                                  const tx_tensor* weight, int reduction, void* workspace, size_t workspace_bytes,
                                  void* stream);
size_t tx_binary_cross_entropy_workspace_bytes(const tx_tensor* out, const tx_tensor* input, const tx_tensor* target,
                                               const tx_tensor* weight, int reduction);

enum { TX_LOSS_MSE = 0, TX_LOSS_L1 = 1, TX_LOSS_SMOOTH_L1 = 2, TX_LOSS_HUBER = 3 };

/* Regression losses (Table 1 "Deep Learning"; the same term-then-reduce shape as
 * the binary_cross_entropy listing of Appendix B.1).  With d = input - target on
 * the broadcast of the two shapes:
 *   MSE d^2;  L1 |d|;
 *   SMOOTH_L1 |d| < beta ? d^2 / (2 beta) : |d| - beta / 2  (param = beta >= 0);
 *   HUBER |d| <= delta ? d^2 / 2 : delta (|d| - delta / 2)  (param = delta > 0);
 * a parameter outside its range, an unknown kind or reduction is TX_ERR_SCALAR.
 * input, target and out have one floating dtype.  reduction NONE: out has the
 * broadcast shape and may alias an operand exactly.  MEAN / SUM: out is 0-dim;
 * terms are formed in fp32 and added in fp32 per thread, binary64 across threads
 * and workgroups; the mean of no elements is NaN, the sum 0.  They need a 16-byte
 * aligned device workspace of tx_loss_workspace_bytes() bytes (0 for NONE). */
tx_status tx_loss(int kind, const tx_tensor* out, const tx_tensor* input, const tx_tensor* target, int reduction, double param,
                  void* workspace, size_t workspace_bytes, void* stream);
size_t tx_loss_workspace_bytes(int kind, const tx_tensor* out, const tx_tensor* input, const tx_tensor* target, int reduction,
                               double param);

/* ------------------------------------------------------------------ reductions
 * (Table 1 "Reduction"; the row mean / variance kernels of the layer_norm
 * listing in Appendix B are the paper's form of the inner-dim case.)
 *
 * Reduce x over dims[0..ndims) (negative dims wrap; ndims == 0 or dims == NULL:
 * all dims).  keepdim keeps reduced dims with size 1.
 *   SUM   bool / integer x -> int64 result (exact, wrapping); float x keeps its
 *         dtype, accumulated in fp32.
 *   MEAN  float only; sum / count; NaN for an empty extent.
 *   PROD  like SUM; one dim or all dims only; empty product = 1.
 *   AMAX  keeps dtype; NaN if any NaN; several dims allowed.
 *   ARGMAX int64 index along the one dim, or flat row-major index over x's
 *         logical shape with no dim; ties -> lowest index; NaN outranks
 *         everything, first NaN wins; bool is TX_ERR_DTYPE.
 *   VAR   float only; sum of squared deviations / max(0, n - correction).
 *   STD   the square root of VAR.
 *   AMIN / ARGMIN  AMAX / ARGMAX with the order reversed (NaN still wins, ties
 *         still go to the lowest index).
 *   ANY / ALL  any input dtype, bool result: some / every element is non-zero
 *         (NaN is non-zero); empty extent: ANY false, ALL true.
 *   LOGSUMEXP  bool / integer input is converted to fp32 (fp32 result); log of the sum of exp(x), computed as a running
 *         (maximum, scaled sum) pair; -inf for an empty or all -inf extent,
 *         +inf if +inf is present, NaN is sticky.
 *   NANSUM / NANMEAN  the sum / mean of the elements that are not NaN (the mean
 *         divides by their count: NaN when there is none); NANSUM of a bool /
 *         integer x is SUM; NANMEAN takes floats only.
 *   COUNT_NONZERO  any dtype, int64 result; a NaN is not zero, -0.0 is.
 *   NORM  the vector p-norm, p passed in `correction`; floats only.  p = 0: the
 *         count of non-zero elements; p = +inf / -inf: the largest / smallest
 *         |x|, NaN if any NaN (an empty extent is TX_ERR_EMPTY_REDUCTION, as it
 *         is for a negative p); p = 2 accumulates squares in binary64, so only
 *         a result beyond the dtype's range overflows; any other p is
 *         (sum |x|^p)^(1/p) in binary64.  A NaN p is TX_ERR_SCALAR.
 * For SUM / MEAN / PROD / VAR / STD / LOGSUMEXP / NANSUM / NANMEAN / NORM on
 * fp16 / bf16 input, out may be fp32.
 * ws / ws_bytes: device scratch of at least tx_reduce_workspace_bytes() for the
 * same arguments (0 when the reduction is not split across workgroups; the
 * data pointers of out / x are not dereferenced by the query). */
tx_status tx_reduce(int op, const tx_tensor* out, const tx_tensor* x, const int64_t* dims, int32_t ndims, int keepdim,
                    double correction, void* ws, size_t ws_bytes, void* stream);
size_t tx_reduce_workspace_bytes(int op, const tx_tensor* out, const tx_tensor* x, const int64_t* dims, int32_t ndims,
                                 int keepdim);

/* tx_reduce for callers that cannot allocate device memory or must not have
 * it allocated on their behalf (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, same kernels and
 * same results as tx_reduce, but the partial results of a reduction that is
 * split across workgroups go to a buffer built into the library instead of a
 * caller workspace.  The call allocates and frees nothing.
 *   - The buffer is TX_REDUCE_STATIC_SCRATCH_BYTES (4 MiB) of device memory per
 *     GPU, part of the loaded library, held until the process ends.  A
 *     reduction whose tx_reduce_workspace_bytes() exceeds it is refused with
 *     TX_ERR_WORKSPACE before any launch (every all-dims reduction needs at
 *     most 32 KiB).
 *   - The buffer belongs to the device that is current when the call is made;
 *     out, x and stream must belong to that device.
 *   - Every call on one GPU shares that GPU's buffer: two calls may overlap
 *     only if they are ordered on one stream; calls on different streams (or
 *     from different threads) that overlap in time race on the partials.
 *     Nothing in the buffer has to start at zero (the first pass writes every
 *     partial the second one reads), so no clearing is done or needed. */
#define TX_REDUCE_STATIC_SCRATCH_BYTES ((size_t)4 << 20)
tx_status tx_reduce_static(int op, const tx_tensor* out, const tx_tensor* x, const int64_t* dims, int32_t ndims,
                           int keepdim, double correction, void* stream);

/* softmax / log_softmax (Table 1 "Deep Learning", the category with the paper's
 * lowest coverage; a row maximum, a row sum and an elementwise pass, the same
 * row skeleton as the layer_norm listing of Appendix B).
 * softmax (is_log == 0) or log_softmax (is_log != 0) of x along `dim`.
 * Float dtypes only; out has x's shape and dtype, or fp32 for a half x.
 * m = max; softmax = exp(x-m)/sum exp(x-m); log_softmax = (x-m) - log sum.
 * A slice that is all -inf, or holds +inf or NaN, is all NaN. */
tx_status tx_softmax(const tx_tensor* out, const tx_tensor* x, int64_t dim, int is_log, void* stream);

/* cumsum (Table 1 "Reduction": the scan member of the category; Section 3.3
 * lists it among the operators whose loop-carried dependence the generated
 * kernels handle with a sequential loop per row).
 * Inclusive prefix sum of x along `dim`.  bool / int32 / int64 x -> int64 out
 * (exact, wrapping); float x keeps its dtype (or fp32 out for a half x),
 * accumulated in fp32.  ws / ws_bytes: device scratch of at least
 * tx_cumsum_workspace_bytes() (tile status words for the single-pass scan; see
 * tx_lookback_status for the one failure that scan can report afterwards). */
tx_status tx_cumsum(const tx_tensor* out, const tx_tensor* x, int64_t dim, void* ws, size_t ws_bytes, void* stream);
size_t tx_cumsum_workspace_bytes(const tx_tensor* out, const tx_tensor* x, int64_t dim);

enum { TX_SCAN_SUM = 0, TX_SCAN_PROD = 1, TX_SCAN_LOGSUMEXP = 2 };

/* Inclusive scan along `dim` with another combining operation; shapes, dim,
 * aliasing and workspace rules as tx_cumsum (TX_SCAN_SUM is tx_cumsum).
 *   PROD       cumprod: dtypes as cumsum (bool / integer x -> int64, wrapping);
 *              floats multiply in binary64 and each prefix is rounded once.
 *   LOGSUMEXP  logcumsumexp: floats only; out[i] = log(sum_{j<=i} exp(x[j])),
 *              carried as (largest exponent m, sum of exp(x - m)) pairs in fp32
 *              with one logarithm per output; -inf
 *              while only -inf has been seen, +inf from the first +inf on, NaN
 *              from the first NaN on.
 * Another code is TX_ERR_SCALAR.  A contiguous `dim` takes the single-pass
 * look-back / row-carry kernels; other layouts one lane per slice. */
tx_status tx_scan(int op, const tx_tensor* out, const tx_tensor* x, int64_t dim, void* ws, size_t ws_bytes, void* stream);
size_t tx_scan_workspace_bytes(int op, const tx_tensor* out, const tx_tensor* x, int64_t dim);

/* ------------------------------------------------------------------ indexing
 * (Table 1 "Indexing & Selection".)  Index tensors are int64 or int32.  By
 * default they are NOT range-checked: an index outside [0, extent) is
 * undefined behaviour (an out-of-bounds access on the device), as on ATen's
 * device backends.  There is no negative-index wrap-around except where a
 * function says so (tx_index_put_, tx_take).
 *
 * Index validation is an opt-in mode.  With it on, tx_gather, tx_index_select,
 * tx_scatter_add_, tx_scatter_reduce_, tx_index_add_, tx_index_put_ and tx_take
 * first run one extra pass over the index tensor(s) on `stream`, synchronise
 * the stream, and return TX_ERR_INDEX - before any data kernel is launched,
 * nothing written - if a value lies outside the valid range ([0, extent), or
 * [-extent, extent) where negative indices wrap); tx_last_error() names the
 * value and its position.  The extra pass and the synchronisation make it a
 * debugging mode: keep it off where time matters and inside graph capture.
 * The switch is per calling thread; its initial state is off, or on when the
 * environment variable TX_VALIDATE_INDICES is set to anything but "0".  The
 * pass keeps its one flag word in the library image (no allocation); calls
 * with validation on are serialised on that word.
 */
void tx_set_index_validation(int on);
int tx_get_index_validation(void);

/* out[i...] = src[i... with coordinate `dim` replaced by index[i...]].
 * index.ndim == src.ndim; index.size(d) <= src.size(d) for d != dim; out has
 * index's shape and src's dtype. */
tx_status tx_gather(const tx_tensor* out, const tx_tensor* src, int64_t dim, const tx_tensor* index, void* stream);

/* out = src with extent `dim` replaced by len(index); slice j of out is slice
 * index[j] of src.  index is 1-D (0-dim counts as length 1). */
tx_status tx_index_select(const tx_tensor* out, const tx_tensor* src, int64_t dim, const tx_tensor* index,
                          void* stream);

/* In place: for every position p of index, self[p with coordinate dim =
 * index[p]] += src[p].  self, index, src have the same ndim; index.size(d) <=
 * src.size(d) for all d and <= self.size(d) for d != dim; self.dtype ==
 * src.dtype.  index may be a stride-0 expanded view.  Integer dtypes use
 * device atomics (exact, order-free); bool ORs.  When the index is a row id
 * broadcast over the trailing dims (at least 4096 rows) and a workspace is
 * given, int32 / int64 rows are instead grouped by destination with the same
 * sort as the float path and added as whole rows, without atomics; without a
 * workspace the call falls back to atomics.  Float dtypes: with
 * deterministic != 0 the contributions are sorted by destination and summed in
 * a fixed order with fp32 accumulation (bitwise reproducible run to run); with
 * deterministic == 0, fp32 uses float atomics (fp16 / bf16 keep the sorted
 * path: 16-bit atomics would round every partial sum).  ws / ws_bytes: device
 * scratch of at least tx_scatter_add_workspace_bytes() for the same arguments
 * (0 for the atomic paths). */
tx_status tx_scatter_add_(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* src,
                          int deterministic, void* ws, size_t ws_bytes, void* stream);
size_t tx_scatter_add_workspace_bytes(const tx_tensor* self, int64_t dim, const tx_tensor* index,
                                      const tx_tensor* src, int deterministic);

/* In place: self[..., index[i], ...] += alpha * source[..., i, ...] along dim.
 * index is 1-D (or 0-dim) int32 / int64 with source.size(dim) entries in
 * [0, self.size(dim)); source has self's shape except along dim and self's
 * dtype.  alpha as in tx_add (a floating alpha with an integer dtype is
 * TX_ERR_SCALAR); integers wrap; bool: self OR (alpha != 0 AND source).  Kernels, determinism and
 * workspace exactly as tx_scatter_add_ with the index broadcast over the other
 * dims: dim 0 with contiguous rows takes the sorted whole-row path. */
tx_status tx_index_add_(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* source, double alpha_f,
                        int64_t alpha_i, int alpha_is_int, int deterministic, void* ws, size_t ws_bytes, void* stream);
size_t tx_index_add_workspace_bytes(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* source,
                                    int deterministic);

enum { TX_SCATTER_SUM = 0, TX_SCATTER_PROD = 1, TX_SCATTER_MEAN = 2, TX_SCATTER_AMAX = 3, TX_SCATTER_AMIN = 4 };

/* In place: every position p of index sends src[p] to self[p with coordinate
 * dim = index[p]]; the values that arrive at an element are combined by
 * `reduce` (TX_SCATTER_*; another code is TX_ERR_SCALAR) with each other and,
 * when include_self != 0, with the element's own value.  Elements that receive
 * nothing keep their bits.  Shapes and dtypes as tx_scatter_add_; bool: SUM
 * and AMAX are OR, PROD and AMIN are AND, MEAN is TX_ERR_DTYPE.  Integers wrap, MEAN divides rounding toward -infinity; floats
 * are combined in binary64 in position order and rounded once; AMAX / AMIN give
 * NaN when a NaN takes part.  Always a sorted path (reproducible run to run):
 * needs a 16-byte aligned workspace of tx_scatter_reduce_workspace_bytes().
 * SUM, AMAX and AMIN over dim 0 with a row id broadcast over contiguous rows
 * take the whole-row kernels of tx_scatter_add_ (sums of floats then in fp32,
 * in sorted source-row order). */
tx_status tx_scatter_reduce_(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* src, int reduce,
                             int include_self, void* ws, size_t ws_bytes, void* stream);
size_t tx_scatter_reduce_workspace_bytes(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* src,
                                         int reduce, int include_self);

/* In place: `nidx` index tensors (int32 / int64; 1 <= nidx <= self.ndim, else
 * TX_ERR_DIM) address the first nidx dims of self; they broadcast together to a
 * shape I, and values (self's dtype) broadcasts to I + self.shape[nidx:].  For
 * every position p of I and coordinate r of the remaining dims,
 * self[idx_0[p], ..., idx_{nidx-1}[p], r] = values[p, r], or += when
 * accumulate != 0.  Negative indices count from the end; indices are not
 * range-checked on the device.  `indices` is a host array of descriptor
 * pointers.  accumulate = 0: when several positions name one element, which of
 * them is kept is unspecified.  accumulate != 0: integers / bool use device
 * atomics (exact); floats sort the destinations and sum each in position order
 * (binary64, reproducible) and need a 16-byte aligned workspace of
 * tx_index_put_workspace_bytes() (0 otherwise). */
tx_status tx_index_put_(const tx_tensor* self, const tx_tensor* const* indices, int32_t nidx, const tx_tensor* values,
                        int accumulate, void* ws, size_t ws_bytes, void* stream);
size_t tx_index_put_workspace_bytes(const tx_tensor* self, const tx_tensor* const* indices, int32_t nidx,
                                    const tx_tensor* values, int accumulate);

/* out[p] = input, read as a 1-D tensor in logical (row-major) order whatever
 * its strides, at index[p]; negative indices count from the end.  out has
 * index's shape and input's dtype; index is int32 / int64.  Indices outside
 * [-numel, numel) are not checked on the device (a non-empty index into an
 * empty input is TX_ERR_INDEX). */
tx_status tx_take(const tx_tensor* out, const tx_tensor* input, const tx_tensor* index, void* stream);

/* searchsorted / bucketize (Table 1, indexing operators): out[p] = the index
 * at which values[p] would be inserted into its sorted sequence so that the
 * order is kept - the first position whose element is >= the value (right =
 * 0) or > the value (right != 0).  A 1-D sorted_sequence serves every value
 * (bucketize's boundaries); otherwise it has the values' rank and leading
 * dims and the rows are searched one by one.  The index comes from bisection
 * of [0, n) with the midpoint start + (end - start) / 2, moving right while
 * !(element >= value) (or !(element > value)): on a sorted sequence without
 * NaN that is the count of elements below (at most) the value; a NaN value
 * lands at n; on unsorted input the result is what these steps give.  All
 * three are device tensors, any strides; the two inputs share one dtype that
 * is not bool (TX_ERR_DTYPE), out is int64 or int32 with the values' shape
 * (TX_ERR_SHAPE) and overlaps neither input (TX_ERR_OVERLAP).  No sorter
 * argument; at most 2^31 values and sequence elements (TX_ERR_UNSUPPORTED). */
tx_status tx_searchsorted(const tx_tensor* out, const tx_tensor* sorted_sequence, const tx_tensor* values, int right, void* stream);

/* Data-dependent output sizes.  The caller passes `out` as a buffer with room
 * for `capacity` results and `count`, a one-element int64 device tensor; the
 * call writes the number of selected elements to `count` and the first
 * min(count, capacity) results to out, in logical (row-major) order (so
 * count > capacity tells the caller the buffer was too small; numel of the
 * input always suffices).  Both need a 16-byte aligned device workspace of
 * tx_*_workspace_bytes() bytes and handle fewer than 2^31 elements.
 *   masked_select: the elements of x, broadcast with the bool mask, where the
 *     mask is true; out is 1-D with x's dtype.
 *   nonzero: the coordinates of the elements of x that are not zero (-0.0 is
 *     zero, a NaN is not); out is int64 [capacity, x.ndim]. */
tx_status tx_masked_select(const tx_tensor* out, const tx_tensor* count, const tx_tensor* x, const tx_tensor* mask,
                           void* workspace, size_t workspace_bytes, void* stream);
size_t tx_masked_select_workspace_bytes(const tx_tensor* out, const tx_tensor* count, const tx_tensor* x,
                                        const tx_tensor* mask);
tx_status tx_nonzero(const tx_tensor* out, const tx_tensor* count, const tx_tensor* x, void* workspace, size_t workspace_bytes,
                     void* stream);
size_t tx_nonzero_workspace_bytes(const tx_tensor* out, const tx_tensor* count, const tx_tensor* x);

/* ------------------------------------------------------------------ shape manipulation
 * (Table 1 "Shape Manipulation": views are the caller's business - a
 * descriptor with other sizes and strides - these are the members that move
 * data.)
 *
 * tx_copy: out = x broadcast to out's shape and converted to out's dtype (clone,
 *   contiguous, to, an expand made real, copy_; cat and stack are copies into
 *   slices of out).  Floating to floating: one rounding.  bool / integer to
 *   floating: through fp32, nearest-even.  Floating to integer: truncated
 *   toward zero (NaN and values outside the target range are outside the
 *   contract).  Anything to bool: value != 0.  int64 to int32 wraps.  Equal
 *   dtypes copy the bits.  out may alias x exactly.
 * tx_flip: out[i] = x[j] with j = size - 1 - i along every listed dim (a dim
 *   listed twice is TX_ERR_DIM).
 * tx_roll: the element at j moves to (j + shift) mod size along every listed
 *   dim; n shifts for n dims; a dim listed twice adds its shifts.
 * tx_tri: upper == 0 tril: out[..., i, j] = x[..., i, j] where j - i <=
 *   diagonal, else 0; upper != 0 triu: where j - i >= diagonal.  At least two
 *   dims (TX_ERR_NDIM).
 * flip / roll / tri: out has x's shape and dtype and may not alias x. */
tx_status tx_copy(const tx_tensor* out, const tx_tensor* x, void* stream);
tx_status tx_flip(const tx_tensor* out, const tx_tensor* x, const int64_t* dims, int32_t ndims, void* stream);
tx_status tx_roll(const tx_tensor* out, const tx_tensor* x, const int64_t* shifts, const int64_t* dims, int32_t n, void* stream);
tx_status tx_tri(const tx_tensor* out, const tx_tensor* x, int64_t diagonal, int upper, void* stream);

/* ------------------------------------------------------------------ host-only helpers */

/* Result dtype and broadcast shape of a binary op (TX_ADD .. TX_TRUNC_DIVIDE). */
tx_status tx_infer_binary(int op, const tx_tensor* a, const tx_tensor* b, int32_t* dtype, int32_t* ndim,
                          int64_t* sizes);
/* Result dtype of where(cond, x, y). */
tx_status tx_infer_where(const tx_tensor* x, const tx_tensor* y, int32_t* dtype);
/* Result dtype of a unary op for an input dtype (negative = error). */
int32_t tx_infer_unary_dtype(int op, int32_t in_dtype);
/* Result dtype of tx_clamp (a TX_* dtype code >= 0) or a negative tx_status. */
int32_t tx_infer_clamp_dtype(int32_t x_dtype, int has_lo, int lo_is_int, int has_hi, int hi_is_int);
/* Result dtype and shape of a reduction. */
tx_status tx_infer_reduce(int op, const tx_tensor* x, const int64_t* dims, int32_t ndims, int keepdim, int32_t* dtype,
                          int32_t* ndim, int64_t* sizes);

/* Name of the kernel path the last call on this thread dispatched to
 * ("" if it launched nothing).  For tests and profiling. */
const char* tx_last_path(void);

/* The single-pass scans (tx_cumsum / tx_scan on paths "scan-lookback*") and the
 * single-pass compaction ("select-fused") make each tile wait for its
 * predecessors' status words.  The wait is bounded (2^24 polls); if it ever
 * gives up, the tile continues with an empty prefix, the kernel still ends, and
 * the error flag in the workspace header is set: the call has long returned
 * TX_OK by then, and its output is wrong.  This query is how a caller finds
 * out: it copies the 16-byte header of `ws` (the workspace that call was given)
 * back on `stream`, synchronises the stream, and returns TX_OK, or
 * TX_ERR_LAUNCH if the flag is set.  A workspace whose last user was not a
 * look-back path carries no header tag and reports TX_OK.  Host-side cost: one
 * small copy and a synchronisation - for tests and for callers that must know,
 * not for the timed path.  What to do on TX_ERR_LAUNCH: run the call again (a
 * predecessor that never publishes means the GPU lost a workgroup, not that
 * the input was bad); the path "scan-carry" needs no waiting at all. */
tx_status tx_lookback_status(const void* ws, void* stream);

/* Force a kernel path by name ("" or NULL = automatic).  Elementwise iterator:
 * "vec", "tile" (reported as "tile" when 16-byte vectors serve, else as
 * "tile-scalar"), "generic"; on the vec path "vec-cached" (plain instead of
 * non-temporal loads), and where every input is a broadcast "vec-wide" /
 * "vec-narrow" (the general vec kernel with four / one vectors per lane instead
 * of the lean broadcast kernel "vec-bcast").  cumsum along a contiguous dim: "scan-lookback"
 * (tile size automatic), "scan-lookback-narrow" (16 KiB tiles), "scan-carry",
 * and "scan-lookback-giveup" (the look-back kernel with a poll limit of zero:
 * every wait gives up at once, for testing tx_lookback_status).
 * Reduction with lanes along the kept dim: "cols-nv1", "cols-nv2", "cols-nv4"
 * (vectors per thread); over rows of 1 to 2 KiB: "rows-wave" (a wave per row
 * instead of half a wave, "rows-half").  Integer scatter_add_: "scatter-atomic" (one atomic
 * per element even when a workspace is given).  scatter_reduce_:
 * "scatter-reduce-sort" (element keys even for a broadcast row index).
 * softmax along a contiguous last dim: "softmax-wave" (a wave per row, for rows
 * of up to 1024 16-byte vectors) and "softmax-row" (a 256-lane workgroup per
 * row, 65 to 4096 vectors) where the other would be chosen.  softmax / cumsum along a
 * non-innermost dim: "softmax-strided", "scan-strided" (one lane per slice
 * instead of the column kernels); "softmax-cols" (the two-read column kernel
 * also where the operated dim is short enough to stay in registers); cumsum along a non-innermost dim whose
 * columns are cut into several tiles: "scan-cols-3pass" (tile sums, their
 * prefixes and the scan as three kernels instead of the single pass with
 * look-back between tiles, "scan-cols-lookback") and
 * "scan-cols-lookback-giveup" (poll limit zero, as above).  layer_norm:
 * "layer-norm-wave" (a wave per row also for rows of 257 to 1024 vectors,
 * which otherwise take a workgroup per row, "layer-norm-row"), "layer-norm-block"
 * (the general workgroup-per-row kernel), "layer-norm-generic" (three passes,
 * any strides).
 * masked_select: "select-fused" (one pass with decoupled look-back instead of
 * the count, offsets and write passes); nonzero: "select-3pass" (those three
 * passes instead of its single pass, "nonzero-fused").  index_put_ without
 * accumulation: "index-put" (one lane per element also where whole dense rows
 * would be copied by "index-put-rows").  binary_cross_entropy sum / mean: "bce-two-pass" (losses into the workspace
 * first; the workspace query then reports that form's size); tx_loss:
 * "loss-two-pass" likewise.  searchsorted: "searchsorted" (every probe from
 * memory, also where the first levels would be walked in LDS).  Requests that a path cannot
 * serve fall back to the automatic choice.  Per calling thread, like
 * tx_last_error and tx_last_path (a thread's forced path affects only the
 * calls that thread makes); meant for A/B profiling. */
void tx_force_path(const char* name);

const char* tx_strerror(tx_status status);
const char* tx_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TXOPS_H */
