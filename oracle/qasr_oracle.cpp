// CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, obviously-correct definition of the integer-only encoder layer of
// "Integer-only Zero-shot Quantization for Efficient Speech Recognition" (Sec. 2.1-2.2):
// symmetric int8 tensors (Eq. 1: q in [-2^(b-1), 2^(b-1)-1], zero-point 0, so padding is the
// integer 0), integer convolution applied directly to the quantised values (Sec. 2.2,
// linearity of Conv / MatMul / ReLU), BatchNorm folded into the preceding convolution
// (Sec. 2.2) which leaves an int32 bias on the accumulator, and a static per-channel dyadic
// rescale m * 2^-s back to int8.  The paper delegates the rescale arithmetic to the
// integer-only schemes it cites; the reading fixed here is
//     v = floor((A*m + 2^(s-1)) / 2^s)       (round half up, i.e. ties toward +infinity)
//     v += residual (int8, already at the output scale; main branch NOT saturated first)
//     y = clamp(v, relu ? 0 : -128, 127)
//
// Only tests, the smoke check and the benchmark's cpu_baseline leg may call this library.
// It shares no code, header or table with the HIP path.  Loops are written in the order
// of the definition (batch, out-channel, out-frame; then in-channel, tap); the only
// parallelism is an OpenMP "for" over (batch, out-channel) pairs.
//
// Pins (tests, CPU-only): brute force against arbitrary-precision Python on tiny shapes,
// float64 library convolution at real shapes (exact below 2^53), one-hot / identity / ones
// closed forms, the (m=2^30, s=30) identity, hand-worked rounding and saturation vectors,
// and the float dequantised product within 1 LSB.  End-to-end encoder bits at full size
// are pinned by composition only.  The quantiser / dequantiser at the two ends of the path
// (bottom of this file) are pinned by hand-worked codes, the round trip over all 255 codes,
// the half-step error bound, odd symmetry and monotonicity, and a float64 recomputation.
#include <cmath>
#include <cstdint>
#include <cstddef>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// floor(v / 2^s) for 1 <= s <= 62, written without shifting a negative value.
inline int64_t floor_div_pow2(int64_t v, int s) {
    const int64_t d = int64_t(1) << s;
    int64_t q = v / d;              // truncates toward zero
    if ((v % d) != 0 && v < 0) q -= 1;
    return q;
}

inline int64_t requant_one(int64_t A, int32_t m, int32_t s) {
    // |A| < 2^31, 0 <= m < 2^31  =>  |A*m| < 2^62 and adding 2^(s-1) <= 2^61 stays in int64.
    return floor_div_pow2(A * int64_t(m) + (int64_t(1) << (s - 1)), s);
}

inline int8_t clamp_out(int64_t v, bool relu) {
    const int64_t lo = relu ? 0 : -128;
    if (v < lo) v = lo;
    if (v > 127) v = 127;
    return int8_t(v);
}

inline int64_t out_len(int64_t Tin, int k, int stride, int dil, int pl, int pr) {
    const int64_t span = Tin + pl + pr - int64_t(dil) * (k - 1) - 1;
    return span < 0 ? 0 : span / stride + 1;
}

// Accumulator of one output element (Sec. 2.2: integer convolution on q_W, q_x),
// cross-correlation (no kernel flip), zero padding, optional int32 bias.
inline int64_t acc_one(const int8_t* xb /* batch item base */, const int8_t* w, const int32_t* bias,
                       int Cin, int64_t Tin, int k, int stride, int dil, int pl, bool depthwise,
                       int co, int64_t to) {
    int64_t A = bias ? int64_t(bias[co]) : 0;
    const int ci_lo = depthwise ? co : 0;
    const int ci_hi = depthwise ? co + 1 : Cin;
    const int cin_g = depthwise ? 1 : Cin;
    for (int ci = ci_lo; ci < ci_hi; ++ci) {
        const int8_t* xr = xb + int64_t(ci) * Tin;
        const int8_t* wr = w + (int64_t(co) * cin_g + (depthwise ? 0 : ci)) * k;
        for (int j = 0; j < k; ++j) {
            const int64_t ti = to * stride - pl + int64_t(j) * dil;
            if (ti >= 0 && ti < Tin) A += int64_t(xr[ti]) * int64_t(wr[j]);
        }
    }
    return A;
}

}  // namespace

extern "C" {

// Threads the OpenMP loops will use (1 when built without OpenMP).
int qasr_oracle_num_threads() {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int64_t qasr_oracle_out_len(int64_t Tin, int k, int stride, int dil, int pl, int pr) {
    return out_len(Tin, k, stride, dil, pl, pr);
}

// Raw accumulators (bias included when given) as int64 [B,Cout,Tout]; for pinning a2-a5.
void qasr_oracle_conv1d_acc(int B, int Cin, int Cout, int64_t Tin, int k, int stride, int dil,
                            int pl, int pr, int groups, int64_t x_batch_stride,
                            const int8_t* x, const int8_t* w, const int32_t* bias, int64_t* acc) {
    const int64_t Tout = out_len(Tin, k, stride, dil, pl, pr);
    const bool dw = groups != 1;
    const int64_t xbs = x_batch_stride ? x_batch_stride : int64_t(Cin) * Tin;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int co = 0; co < Cout; ++co)
            for (int64_t to = 0; to < Tout; ++to)
                acc[(int64_t(b) * Cout + co) * Tout + to] =
                    acc_one(x + b * xbs, w, bias, Cin, Tin, k, stride, dil, pl, dw, co, to);
}

// One layer: conv -> +bias -> dyadic requant -> +residual -> clamp (ReLU if flags&1).
// Returns the number of output elements whose accumulator left the int32 range
// (the GPU path would wrap there; the caller's contract is that this is 0).
int64_t qasr_oracle_conv1d_int8(int B, int Cin, int Cout, int64_t Tin, int k, int stride, int dil,
                                int pl, int pr, int groups, int64_t x_batch_stride,
                                int64_t y_batch_stride, uint32_t flags,
                                const int8_t* x, const int8_t* w, const int32_t* bias,
                                const int32_t* m, const int32_t* s, const int8_t* residual,
                                int8_t* y) {
    const int64_t Tout = out_len(Tin, k, stride, dil, pl, pr);
    const bool dw = groups != 1;
    const bool relu = (flags & 1u) != 0;
    const int64_t xbs = x_batch_stride ? x_batch_stride : int64_t(Cin) * Tin;
    const int64_t ybs = y_batch_stride ? y_batch_stride : int64_t(Cout) * Tout;
    int64_t overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(+ : overflow)
    for (int b = 0; b < B; ++b)
        for (int co = 0; co < Cout; ++co)
            for (int64_t to = 0; to < Tout; ++to) {
                const int64_t A = acc_one(x + b * xbs, w, bias, Cin, Tin, k, stride, dil, pl, dw, co, to);
                if (A < INT32_MIN || A > INT32_MAX) ++overflow;
                int64_t v = requant_one(A, m[co], s[co]);
                const int64_t o = b * ybs + int64_t(co) * Tout + to;
                if (residual) v += int64_t(residual[o]);
                y[o] = clamp_out(v, relu);
            }
    return overflow;
}

// The same layer with several residual operands (the dense-residual wiring of the Jasper family
// named in Sec. 3: a block receives the projected inputs of all earlier blocks).  The paper does
// not say how the operands combine in integers; the reading: every operand is int8 at the output
// scale, all are added to the unsaturated requantised value, one clamp follows:
//     v = requant(A) + sum_r residual_r ;  y = clamp(v)
// (n_res = 1 is the layer above; saturating after each addition would differ, a pin separates them).
int64_t qasr_oracle_conv1d_int8_multi(int B, int Cin, int Cout, int64_t Tin, int k, int stride, int dil,
                                      int pl, int pr, int groups, int64_t x_batch_stride,
                                      int64_t y_batch_stride, uint32_t flags,
                                      const int8_t* x, const int8_t* w, const int32_t* bias,
                                      const int32_t* m, const int32_t* s,
                                      const int8_t* const* residuals, int n_res, int8_t* y) {
    const int64_t Tout = out_len(Tin, k, stride, dil, pl, pr);
    const bool dw = groups != 1;
    const bool relu = (flags & 1u) != 0;
    const int64_t xbs = x_batch_stride ? x_batch_stride : int64_t(Cin) * Tin;
    const int64_t ybs = y_batch_stride ? y_batch_stride : int64_t(Cout) * Tout;
    int64_t overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(+ : overflow)
    for (int b = 0; b < B; ++b)
        for (int co = 0; co < Cout; ++co)
            for (int64_t to = 0; to < Tout; ++to) {
                const int64_t A = acc_one(x + b * xbs, w, bias, Cin, Tin, k, stride, dil, pl, dw, co, to);
                if (A < INT32_MIN || A > INT32_MAX) ++overflow;
                int64_t v = requant_one(A, m[co], s[co]);
                const int64_t o = b * ybs + int64_t(co) * Tout + to;
                for (int r = 0; r < n_res; ++r) v += int64_t(residuals[r][o]);
                y[o] = clamp_out(v, relu);
            }
    return overflow;
}

// Standalone epilogue: A = acc + bias, then exactly the last four steps above.
void qasr_oracle_requant(const int32_t* acc, int B, int C, int64_t T, const int32_t* bias,
                         const int32_t* m, const int32_t* s, const int8_t* residual,
                         uint32_t flags, int8_t* y) {
    const bool relu = (flags & 1u) != 0;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < C; ++c)
            for (int64_t t = 0; t < T; ++t) {
                const int64_t o = (int64_t(b) * C + c) * T + t;
                const int64_t A = int64_t(acc[o]) + (bias ? int64_t(bias[c]) : 0);
                int64_t v = requant_one(A, m[c], s[c]);
                if (residual) v += int64_t(residual[o]);
                y[o] = clamp_out(v, relu);
            }
}

// Scalar requant (pre-clamp, no residual), exposed so tests can probe single values.
int64_t qasr_oracle_requant_scalar(int64_t A, int32_t m, int32_t s) { return requant_one(A, m, s); }

// ---- the steps either side of the integer path (Sec. 2.1, Eq. 1 and the sentence after it)
//
// Quantiser  q = Q(x, b, S) = Int(clip(x, -alpha, alpha) / S),  S = alpha / (2^(b-1) - 1),  b = 8,
// so q lies in [-127, 127].  The paper calls Int "the round operation" and fixes no precision;
// the reading taken here: single precision throughout (the features are float32), S computed
// once as alpha / 127 in float32, an IEEE division per element, and Int = round to nearest with
// ties to even (the default rounding of the floating-point environment).  A NaN feature has no
// defined code; it is mapped to 0.
void qasr_oracle_quantize(const float* x, int64_t n, float alpha, int8_t* q) {
    const float S = alpha / 127.0f;
    for (int64_t i = 0; i < n; ++i) {
        float v = x[i];
        if (v != v) { q[i] = 0; continue; }
        if (v > alpha) v = alpha;            // clip(x, -alpha, alpha)
        if (v < -alpha) v = -alpha;
        const float u = v / S;
        q[i] = (int8_t)std::nearbyintf(u);   // |u| <= 127 (+ at most one rounding of the division, still 127 after Int)
    }
}

// Dequantiser  x~ = DQ(q, S) = S * q  (one float32 multiplication).
void qasr_oracle_dequantize(const int8_t* q, int64_t n, float S, float* x) {
    for (int64_t i = 0; i < n; ++i) x[i] = S * (float)q[i];
}


// ---- integer-only non-linear activations (Sec. 2.2, last sentence; Sec. 3, first paragraph)
//
// The paper states that Sigmoid, Softmax and Swish are computed with integer arithmetic through
// second-order polynomials, by the procedure of the integer-only BERT work it cites, and gives no
// formula of its own.  The reading fixed here restates that published procedure:
//
//   exp on x <= 0:  x = -z ln2 + p with p in (-ln2, 0], exp(x) = 2^-z exp(p), and
//                   exp(p) ~ 0.3585 (p + 1.353)^2 + 0.344 on that interval.
//   On integers r <= 0 at scale S' (x = S' r), with the host-side constants
//       q_ln2 = floor(ln2 / S'),  q_b = floor(1.353 / S'),  q_c = floor(0.344 / (0.3585 S'^2)):
//       z = floor(-r / q_ln2),  p = r + z q_ln2,  L = (p + q_b)^2 + q_c,  E = floor(L / 2^z)
//   (E = 0 once z > 62), so that exp(S' r) ~ 0.3585 S'^2 E.
//
//   An int8 code at scale S is first refined to scale S' = S / 2^u (r = q 2^u, exact), because the
//   floors in the constants are coarse at an 8-bit step.
//
//   Sigmoid is the two-way softmax of (x, 0), which needs only exp of -|x|:
//       E = iexp(-|q| 2^u),  E0 = iexp(0) = q_b^2 + q_c,
//       sigma_q = floor((q >= 0 ? E0 : E) 2^15 / (E0 + E))          in [0, 2^15], scale 2^-15.
//   Swish(x) = x sigmoid(x) and GLU(a, g) = a sigmoid(g) are integer products with that code; all
//   three go back to int8 through the same dyadic rescale as a layer (round half up, one (m, s)
//   per tensor) and the clamp to [-128, 127]:
//       sigmoid: v = sigma_q(q);  swish: v = q sigma_q(q);  glu: v = a sigma_q(g).
//   GLU splits the channel axis in halves, the first half is the value, the second the gate.
//
//   Softmax over a row of int32 logits at scale S (refined by u as well):
//       r_i = (q_i - max_j q_j) 2^u,  E_i = iexp(r_i),  y_i = min(127, floor(E_i 2^7 / sum_j E_j)),
//   probabilities at scale 2^-7 in int8.
//
// Pins (tests, CPU-only): the real polynomial against exp on (-ln2, 0] within 2.2e-3
// (its three-digit coefficients); iexp against float exp, its exact halving per q_ln2 and monotonicity; the sigmoid code
// against the float function over all 256 codes, its value at 0 and the complement identity;
// swish / glu / sigmoid outputs within one code of the rounded float function (all 256 codes, all
// 65536 pairs); softmax against the float function, shift invariance, the uniform row's closed
// form, the one-hot limit; hand-worked values at S = 0.1.
namespace {

struct IExp { int u; int64_t q_ln2, q_b, q_c; };

inline int64_t iexp_one(int64_t r, const IExp& c) {          // r <= 0
    const int64_t z = (-r) / c.q_ln2;                          // floor: both operands non-negative
    const int64_t p = r + z * c.q_ln2;                         // in (-q_ln2, 0]
    const int64_t L = (p + c.q_b) * (p + c.q_b) + c.q_c;
    return z > 62 ? 0 : L >> z;                                // L >= 0: the shift is floor(L / 2^z)
}

inline int64_t sigmoid_code_one(int q, const IExp& c) {
    const int64_t a = q < 0 ? -int64_t(q) : int64_t(q);
    const int64_t E = iexp_one(-(a * (int64_t(1) << c.u)), c);
    const int64_t E0 = c.q_b * c.q_b + c.q_c;
    const int64_t num = q >= 0 ? E0 : E;
    return (num << 15) / (E0 + E);                             // floor: non-negative operands
}

}  // namespace

// Host-side constants from the real scale (double precision, floor).  Returns 0, or -1 if the
// scale is unusable (not finite, not positive, u outside [0, 16], q_ln2 < 1 or q_b >= 2^24).
int qasr_oracle_iexp_constants(double S, int u, int64_t* out /* q_ln2, q_b, q_c */) {
    if (!(S > 0.0) || !std::isfinite(S) || u < 0 || u > 16) return -1;
    const double Sr = S / double(int64_t(1) << u);
    const double ln2 = 0.693147180559945309417232121458;
    const double ql = std::floor(ln2 / Sr), qb = std::floor(1.353 / Sr);
    const double qc = std::floor(0.344 / (0.3585 * Sr * Sr));
    if (!(ql >= 1.0) || !(qb < 16777216.0)) return -1;
    out[0] = int64_t(ql); out[1] = int64_t(qb); out[2] = int64_t(qc);
    return 0;
}

int64_t qasr_oracle_iexp(int64_t r, int u, int64_t q_ln2, int64_t q_b, int64_t q_c) {
    return iexp_one(r, IExp{u, q_ln2, q_b, q_c});
}

int64_t qasr_oracle_sigmoid_code(int q, int u, int64_t q_ln2, int64_t q_b, int64_t q_c) {
    return sigmoid_code_one(q, IExp{u, q_ln2, q_b, q_c});
}

// kind: 1 sigmoid, 2 swish, 3 glu.  x [B, C (2C for glu), T] with batch stride xbs, y [B, C, T]
// with batch stride ybs (elements).
void qasr_oracle_act(int kind, const int8_t* x, int B, int C, int64_t T, int64_t xbs, int64_t ybs,
                     int u, int64_t q_ln2, int64_t q_b, int64_t q_c, int32_t m, int32_t s, int8_t* y) {
    const IExp c{u, q_ln2, q_b, q_c};
    for (int b = 0; b < B; ++b)
        for (int ch = 0; ch < C; ++ch)
            for (int64_t t = 0; t < T; ++t) {
                const int a = x[b * xbs + int64_t(ch) * T + t];
                int64_t v;
                if (kind == 1) v = sigmoid_code_one(a, c);
                else if (kind == 2) v = int64_t(a) * sigmoid_code_one(a, c);
                else v = int64_t(a) * sigmoid_code_one(x[b * xbs + (int64_t(C) + ch) * T + t], c);
                y[b * ybs + int64_t(ch) * T + t] = clamp_out(requant_one(v, m, s), false);
            }
}

void qasr_oracle_softmax(const int32_t* x, int64_t rows, int64_t L, int u, int64_t q_ln2, int64_t q_b,
                         int64_t q_c, int8_t* y) {
    const IExp c{u, q_ln2, q_b, q_c};
    for (int64_t i = 0; i < rows; ++i) {
        const int32_t* xr = x + i * L;
        int64_t mx = xr[0];
        for (int64_t j = 1; j < L; ++j) if (xr[j] > mx) mx = xr[j];
        const int64_t refine = int64_t(1) << c.u;                 // r_i = (q_i - max) 2^u, a product: the
        int64_t sum = 0;                                           // difference is negative, never shifted
        for (int64_t j = 0; j < L; ++j) sum += iexp_one((int64_t(xr[j]) - mx) * refine, c);
        for (int64_t j = 0; j < L; ++j) {
            const int64_t E = iexp_one((int64_t(xr[j]) - mx) * refine, c);
            const int64_t p = (E << 7) / sum;
            y[i * L + j] = int8_t(p > 127 ? 127 : p);
        }
    }
}


// ---- offline calibration helpers (Sec. 2.1: S, and so alpha, is pre-computed; Sec. 3.1: the
// min/max values seen on the calibration data are the clipping range; Sec. 2.2: BatchNorm is
// folded into the preceding convolution)
//
// Observer: running minimum and maximum of a float32 tensor, NaNs skipped; mm[0] and mm[1] hold
// the extremes seen so far (start them at +inf / -inf).  The clipping range of the symmetric
// quantiser of Eq. 1 is then alpha = max(-min, max).
void qasr_oracle_minmax(const float* x, int64_t n, float* mm) {
    for (int64_t i = 0; i < n; ++i) {
        const float v = x[i];
        if (v != v) continue;
        if (v < mm[0]) mm[0] = v;
        if (v > mm[1]) mm[1] = v;
    }
}

// Dyadic form of a positive real multiplier M (the ratio S_w S_x / S_y of a layer): the integer
// pair with 2^30 <= m < 2^31 and m 2^-s nearest to M,
//     s = 30 - floor(log2 M),  m = round(M 2^s)   (and m = 2^31 carries into m = 2^30, s - 1).
// Returns -1 if M is not positive and finite or s would leave [1, 62].
int qasr_oracle_dyadic(double M, int32_t* m, int32_t* s) {
    if (!(M > 0.0) || !std::isfinite(M)) return -1;
    int e;
    const double f = std::frexp(M, &e);              // M = f 2^e, 1/2 <= f < 1
    int64_t mi = (int64_t)std::nearbyint(std::ldexp(f, 31));   // f 2^31 in [2^30, 2^31]
    int sh = 31 - e;
    if (mi == (int64_t(1) << 31)) { mi >>= 1; --sh; }
    if (sh < 1 || sh > 62) return -1;
    *m = (int32_t)mi; *s = sh;
    return 0;
}

// Fold a BatchNorm into the convolution before it and quantise the result for the integer layer.
// Float model:  y = gamma (conv(x, w) + b - mu) / sqrt(var + eps) + beta.  Per output channel c:
//     f   = gamma / sqrt(var + eps)                      float32, each operation rounded once
//     w'  = w f            b' = (b - mu) f + beta        float32, each operation rounded once
//     S_w = max |w'| / 127                                (per-channel symmetric range, Eq. 1)
//     q_w = Int(w' / S_w)                                 round to nearest, ties to even
//     B   = Int(b' / (S_w S_x))                           int32 bias at the accumulator's scale (double)
//     (m, s) = dyadic(S_w S_x / S_y)                      (double)
// A channel whose folded weights are all zero gets S_w = 1, q_w = 0.  Returns the number of
// channels whose multiplier has no dyadic form in range or whose bias leaves int32 (0 = fine).
int qasr_oracle_fold_quantize(const float* w, const float* b /* or null */, const float* gamma,
                              const float* beta, const float* mu, const float* var, float eps,
                              int Cout, int64_t per /* Cin/groups * k */, float S_x, float S_y,
                              int8_t* qw, int32_t* bias_q, int32_t* m, int32_t* s, float* S_w_out) {
    int bad = 0;
    for (int c = 0; c < Cout; ++c) {
        const float den = std::sqrt(var[c] + eps);
        const float f = gamma[c] / den;
        float amax = 0.0f;
        for (int64_t i = 0; i < per; ++i) {
            const float wf = w[c * per + i] * f;
            const float a = wf < 0.0f ? -wf : wf;
            if (a > amax) amax = a;
        }
        const float Sw = amax > 0.0f ? amax / 127.0f : 1.0f;
        for (int64_t i = 0; i < per; ++i) {
            const float wf = w[c * per + i] * f;
            qw[c * per + i] = (int8_t)std::nearbyintf(wf / Sw);
        }
        const float b0 = b ? b[c] : 0.0f;
        const float d = b0 - mu[c];
        const float t = d * f;
        const float bf = t + beta[c];
        const double acc_scale = (double)Sw * (double)S_x;
        const double bq = std::nearbyint((double)bf / acc_scale);
        if (!(bq >= -2147483648.0 && bq <= 2147483647.0)) { ++bad; bias_q[c] = 0; }
        else bias_q[c] = (int32_t)bq;
        if (qasr_oracle_dyadic(acc_scale / (double)S_y, &m[c], &s[c]) != 0) { ++bad; m[c] = 0; s[c] = 1; }
        S_w_out[c] = Sw;
    }
    return bad;
}

}  // extern "C"
