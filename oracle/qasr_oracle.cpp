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

}  // extern "C"
