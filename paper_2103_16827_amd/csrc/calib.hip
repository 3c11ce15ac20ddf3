// Offline calibration helpers (paper Sec. 2.1: the scale S, and so the clipping range, is
// pre-computed; Sec. 3.1: the min/max values seen on the calibration data are that range;
// Sec. 2.2: BatchNorm is folded into the preceding convolution).  They run once per model, not per
// utterance; they are on the GPU because the calibration activations and the float weights are.
//
//  - observer: running (min, max) of a float32 tensor, NaNs skipped; memory-bound (4 bytes per
//    element): 16-byte loads, grid-stride, one compare-and-swap per workgroup and extreme at the
//    end (a retry means another workgroup moved the extreme; at most one retry per workgroup of
//    the grid).
//  - BatchNorm folding + quantisation, one workgroup per output channel:
//        f = gamma / sqrt(var + eps);  w' = w f;  b' = (b - mean) f + beta     float32, every operation
//                                                                              rounded once (no fusion)
//        S_w = max|w'| / 127 (1 if the channel is all zero);  q_w = Int(w' / S_w)   ties to even
//        bias = Int(b' / (S_w S_x))  int32;  (m, s) = dyadic form of S_w S_x / S_y       (double)
//    A channel whose bias leaves int32 or whose multiplier has no dyadic form with 1 <= s <= 62
//    gets bias 0 / (m, s) = (0, 1) and is counted in *bad_count.
#include "kernels.hpp"

#include <cmath>

// every float operation below is rounded on its own, as written: no multiply-add fusion
#pragma clang fp contract(off)

namespace qasr {

namespace {

__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const float w = __shfl_xor(v, o);
    v = w < v ? w : v;
  }
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const float w = __shfl_xor(v, o);
    v = w > v ? w : v;
  }
  return v;
}

__device__ __forceinline__ void atomic_min_float(float* addr, float v) {
  float old = *addr;
  while (v < old) {                                    // false for a NaN in *addr: the loop ends
    const uint32_t seen = atomicCAS(reinterpret_cast<unsigned int*>(addr), __float_as_uint(old), __float_as_uint(v));
    if (seen == __float_as_uint(old)) break;
    old = __uint_as_float(seen);
  }
}
__device__ __forceinline__ void atomic_max_float(float* addr, float v) {
  float old = *addr;
  while (v > old) {
    const uint32_t seen = atomicCAS(reinterpret_cast<unsigned int*>(addr), __float_as_uint(old), __float_as_uint(v));
    if (seen == __float_as_uint(old)) break;
    old = __uint_as_float(seen);
  }
}

__global__ __launch_bounds__(256) void minmax_kernel(const float* __restrict__ x, size_t n, float* mm, int vec_ok) {
  __shared__ float sh[8];
  float lo = INFINITY, hi = -INFINITY;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n4 = vec_ok ? n / 4 : 0;
  for (size_t i = tid; i < n4; i += stride) {
    const float4 v = reinterpret_cast<const float4*>(x)[i];
    const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {                      // comparisons are false for a NaN: it is skipped
      lo = e[k] < lo ? e[k] : lo;
      hi = e[k] > hi ? e[k] : hi;
    }
  }
  for (size_t i = 4 * n4 + tid; i < n; i += stride) {
    const float v = x[i];
    lo = v < lo ? v : lo;
    hi = v > hi ? v : hi;
  }
  lo = wave_min(lo);
  hi = wave_max(hi);
  if ((threadIdx.x & 63) == 0) { sh[threadIdx.x >> 6] = lo; sh[4 + (threadIdx.x >> 6)] = hi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) {
      lo = sh[w] < lo ? sh[w] : lo;
      hi = sh[4 + w] > hi ? sh[4 + w] : hi;
    }
    atomic_min_float(mm, lo);
    atomic_max_float(mm + 1, hi);
  }
}

// (m, s) with 2^30 <= m < 2^31 and m 2^-s nearest to M; false if M is not positive and finite or s
// would leave [1, 62]
__host__ __device__ inline bool dyadic_of(double M, int32_t& m, int32_t& s) {
  if (!(M > 0.0) || !(M < INFINITY)) return false;
  int e;
  const double f = frexp(M, &e);                      // M = f 2^e, 1/2 <= f < 1
  long long mi = (long long)rint(ldexp(f, 31));
  int sh = 31 - e;
  if (mi == (1ll << 31)) { mi >>= 1; --sh; }
  if (sh < 1 || sh > 62) return false;
  m = (int32_t)mi;
  s = sh;
  return true;
}

__global__ __launch_bounds__(256) void fold_quantize_kernel(const float* __restrict__ w, const float* __restrict__ b,
                                                            const float* __restrict__ gamma, const float* __restrict__ beta,
                                                            const float* __restrict__ mean, const float* __restrict__ var,
                                                            float eps, int64_t per, float S_x, float S_y,
                                                            int8_t* __restrict__ qw, int32_t* __restrict__ bias_q,
                                                            int32_t* __restrict__ m, int32_t* __restrict__ s,
                                                            float* __restrict__ S_w, int32_t* bad_count) {
  __shared__ float sh[4];
  const int c = blockIdx.x;
  const float f = __fdiv_rn(gamma[c], sqrtf(__fadd_rn(var[c], eps)));   // sqrtf: correctly rounded (the _rn intrinsic is the approximate one)
  const float* wc = w + (int64_t)c * per;
  float amax = 0.0f;
  for (int64_t i = threadIdx.x; i < per; i += 256) {
    const float a = fabsf(__fmul_rn(wc[i], f));
    amax = a > amax ? a : amax;
  }
  amax = wave_max(amax);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
  const float Sw = amax > 0.0f ? __fdiv_rn(amax, 127.0f) : 1.0f;
  int8_t* qc = qw + (int64_t)c * per;
  for (int64_t i = threadIdx.x; i < per; i += 256) qc[i] = (int8_t)rintf(__fdiv_rn(__fmul_rn(wc[i], f), Sw));
  if (threadIdx.x == 0) {
    int bad = 0;
    const float bf = __fadd_rn(__fmul_rn(__fsub_rn(b ? b[c] : 0.0f, mean[c]), f), beta[c]);
    const double acc_scale = __dmul_rn((double)Sw, (double)S_x);
    const double bq = rint(__ddiv_rn((double)bf, acc_scale));
    if (bq >= -2147483648.0 && bq <= 2147483647.0) bias_q[c] = (int32_t)bq;
    else { bias_q[c] = 0; ++bad; }
    int32_t mc, sc;
    if (dyadic_of(__ddiv_rn(acc_scale, (double)S_y), mc, sc)) { m[c] = mc; s[c] = sc; }
    else { m[c] = 0; s[c] = 1; ++bad; }
    if (S_w) S_w[c] = Sw;
    if (bad && bad_count) atomicAdd(bad_count, bad);
  }
}

}  // namespace

bool dyadic_from_scale(double M, int32_t& m, int32_t& s) { return dyadic_of(M, m, s); }

hipError_t launch_minmax(const float* x, size_t n, float* mm, hipStream_t st) {
  const int vec_ok = (uintptr_t)x % 16 == 0 ? 1 : 0;
  const size_t blocks = (n / 4 + 255) / 256;
  const unsigned grid = (unsigned)(blocks < 1 ? 1 : (blocks > 2048 ? 2048 : blocks));
  return launch_kernel(minmax_kernel, dim3(grid), dim3(256), 0, st, x, n, mm, vec_ok);
}

hipError_t launch_fold_quantize(const float* w, const float* b, const float* gamma, const float* beta, const float* mean,
                                const float* var, float eps, int32_t Cout, int64_t per, float S_x, float S_y, int8_t* qw,
                                int32_t* bias_q, int32_t* m, int32_t* s, float* S_w, int32_t* bad_count, hipStream_t st) {
  return launch_kernel(fold_quantize_kernel, dim3((unsigned)Cout), dim3(256), 0, st, w, b, gamma, beta, mean, var, eps, per,
                       S_x, S_y, qw, bias_q, m, s, S_w, bad_count);
}

}  // namespace qasr
