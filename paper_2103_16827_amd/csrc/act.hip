// Integer-only non-linear activations (paper Sec. 2.2, last sentence, and Sec. 3, first paragraph:
// Sigmoid, Softmax and Swish go through second-order polynomials so that no floating point is
// executed).  The arithmetic, all of it on integers:
//
//   exp of r <= 0 at scale S' (three host-side constants q_ln2, q_b, q_c):
//       z = floor(-r / q_ln2),  p = r + z q_ln2,  E = floor(((p + q_b)^2 + q_c) / 2^z)   (0 for z > 62)
//   an int8 code q is refined to r = q 2^u first;
//   sigmoid code (two-way softmax of (x, 0)), 15 fraction bits:
//       E = iexp(-|q| 2^u),  E0 = q_b^2 + q_c,  sigma_q = floor((q >= 0 ? E0 : E) 2^15 / (E0 + E))
//   sigmoid: v = sigma_q(q);  swish: v = q sigma_q(q);  GLU: v = a sigma_q(g)  (value = first half
//   of the channels, gate = second half);  y = clamp(floor((v m + 2^(s-1)) / 2^s), -128, 127);
//   softmax of a row of int32 logits: r_i = (q_i - max q) 2^u, y_i = min(127, floor(E_i 2^7 / sum E)).
//
// Elementwise kernels: an int8 code has 256 values, so every workgroup first evaluates the integer
// formulas once per code (thread t takes code t - 128: two 64-bit divisions) into a table in LDS
// (the final int8 for sigmoid and swish, the 16-bit sigmoid code for GLU), then streams the
// tensor through it, 16 bytes per lane and access.  The pass is memory-bound (2 bytes per element,
// 3 for GLU); the table costs each workgroup a few hundred cycles once.
//
// Softmax: one workgroup per row, three passes over the row (maximum, sum of exponentials,
// quotients) with 64-bit integer arithmetic per element; the row stays in cache between passes.
#include "kernels.hpp"

namespace qasr {

namespace {

constexpr int kSigmoidBits = 15;

__device__ __forceinline__ long long iexp_dev(long long r, const ActParams& c) {        // r <= 0
  const unsigned long long nr = (unsigned long long)(-r);
  const unsigned long long z = nr / (unsigned long long)c.q_ln2;
  const long long p = r + (long long)z * c.q_ln2;
  const long long L = (p + c.q_b) * (p + c.q_b) + c.q_c;
  return z > 62 ? 0 : (L >> z);
}

__device__ __forceinline__ int32_t sigmoid_code_dev(int q, const ActParams& c) {
  const long long a = q < 0 ? -(long long)q : (long long)q;
  const long long E = iexp_dev(-(a << c.u), c);
  const long long E0 = c.q_b * c.q_b + c.q_c;
  const unsigned long long num = (unsigned long long)(q >= 0 ? E0 : E) << kSigmoidBits;
  return (int32_t)(num / (unsigned long long)(E0 + E));
}

__device__ __forceinline__ int32_t rescale_clamp(int32_t v, int32_t m, int32_t s) {
  long long w = ((long long)v * (long long)m + (1ll << (s - 1))) >> s;
  w = w > 127 ? 127 : w;
  w = w < -128 ? -128 : w;
  return (int32_t)w;
}

// x, y: [B][C T] int8 per batch item (strides xbs, ybs); grid = (blocks, B)
__global__ __launch_bounds__(256) void act_unary_kernel(ActParams c, const int8_t* x, int8_t* y,
                                                        int64_t n, int64_t xbs, int64_t ybs, int vec_ok) {
  __shared__ uint8_t lut[256];
  {
    const int q = (int)threadIdx.x - 128;
    const int32_t sg = sigmoid_code_dev(q, c);
    lut[threadIdx.x] = (uint8_t)rescale_clamp(c.kind == 2 ? q * sg : sg, c.m, c.s);
  }
  __syncthreads();
  const int8_t* xb = x + (int64_t)blockIdx.y * xbs;
  int8_t* yb = y + (int64_t)blockIdx.y * ybs;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n16 = vec_ok ? n / 16 : 0;
  for (int64_t i = tid; i < n16; i += stride) {
    const uint4 v = reinterpret_cast<const uint4*>(xb)[i];
    const uint32_t in[4] = {v.x, v.y, v.z, v.w};
    uint32_t out[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const uint32_t w = in[d] ^ 0x80808080u;                 // code + 128 in every byte
      out[d] = (uint32_t)lut[w & 0xffu] | ((uint32_t)lut[(w >> 8) & 0xffu] << 8) |
               ((uint32_t)lut[(w >> 16) & 0xffu] << 16) | ((uint32_t)lut[w >> 24] << 24);
    }
    reinterpret_cast<uint4*>(yb)[i] = make_uint4(out[0], out[1], out[2], out[3]);
  }
  for (int64_t i = 16 * n16 + tid; i < n; i += stride) yb[i] = (int8_t)lut[(uint8_t)xb[i] ^ 0x80u];
}

// x: [B][2 n] (value half, gate half), y: [B][n]
__global__ __launch_bounds__(256) void act_glu_kernel(ActParams c, const int8_t* x, int8_t* y,
                                                      int64_t n, int64_t xbs, int64_t ybs, int vec_ok) {
  __shared__ uint16_t lut[256];
  lut[threadIdx.x] = (uint16_t)sigmoid_code_dev((int)threadIdx.x - 128, c);       // 0 .. 2^15
  __syncthreads();
  const int8_t* xa = x + (int64_t)blockIdx.y * xbs;
  const int8_t* xg = xa + n;
  int8_t* yb = y + (int64_t)blockIdx.y * ybs;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n16 = vec_ok ? n / 16 : 0;
  const int32_t m = c.m, s = c.s;
  for (int64_t i = tid; i < n16; i += stride) {
    const uint4 va = reinterpret_cast<const uint4*>(xa)[i];
    const uint4 vg = reinterpret_cast<const uint4*>(xg)[i];
    const uint32_t a4[4] = {va.x, va.y, va.z, va.w}, g4[4] = {vg.x, vg.y, vg.z, vg.w};
    uint32_t out[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const uint32_t g = g4[d] ^ 0x80808080u;
      uint32_t pk = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int32_t a = (int32_t)(int8_t)(a4[d] >> (8 * e));
        const int32_t sg = (int32_t)lut[(g >> (8 * e)) & 0xffu];
        pk |= ((uint32_t)rescale_clamp(a * sg, m, s) & 0xffu) << (8 * e);
      }
      out[d] = pk;
    }
    reinterpret_cast<uint4*>(yb)[i] = make_uint4(out[0], out[1], out[2], out[3]);
  }
  for (int64_t i = 16 * n16 + tid; i < n; i += stride)
    yb[i] = (int8_t)rescale_clamp((int32_t)xa[i] * (int32_t)lut[(uint8_t)xg[i] ^ 0x80u], m, s);
}

__device__ __forceinline__ long long wg_reduce(long long v, bool is_max, long long* sh) {
  // 256 threads: butterfly inside each wave, then the four wave results through LDS
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const int lo = __shfl_xor((int)(uint32_t)(unsigned long long)v, o);
    const int hi = __shfl_xor((int)(uint32_t)((unsigned long long)v >> 32), o);
    const long long w = (long long)(((unsigned long long)(uint32_t)hi << 32) | (uint32_t)lo);
    v = is_max ? (w > v ? w : v) : v + w;
  }
  __syncthreads();                                   // sh may still be read from the previous use
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  const long long a = sh[0], b = sh[1], c = sh[2], d = sh[3];
  return is_max ? max(max(a, b), max(c, d)) : a + b + c + d;
}

__global__ __launch_bounds__(256) void softmax_kernel(ActParams c, const int32_t* __restrict__ x, int64_t rows, int32_t L,
                                                      int8_t* __restrict__ y) {
  __shared__ long long sh[4];
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
    const int32_t* xr = x + row * L;
    int8_t* yr = y + row * L;
    long long mx = INT32_MIN;
    for (int j = threadIdx.x; j < L; j += 256) mx = max(mx, (long long)xr[j]);
    mx = wg_reduce(mx, true, sh);
    long long sum = 0;
    for (int j = threadIdx.x; j < L; j += 256) sum += iexp_dev(((long long)xr[j] - mx) * (1ll << c.u), c);
    sum = wg_reduce(sum, false, sh);
    for (int j = threadIdx.x; j < L; j += 256) {
      const unsigned long long E = (unsigned long long)iexp_dev(((long long)xr[j] - mx) * (1ll << c.u), c);
      const unsigned long long p = (E << 7) / (unsigned long long)sum;      // sum >= E0 > 0 (the maximum's own term)
      yr[j] = (int8_t)(p > 127 ? 127 : p);
    }
  }
}

}  // namespace

hipError_t launch_act(const ActParams& c, const int8_t* x, int8_t* y, int32_t B, int64_t n, int64_t xbs, int64_t ybs,
                      hipStream_t st) {
  // n = C*T outputs per batch item
  const bool glu = c.kind == 3;
  const int vec_ok = ((uintptr_t)x % 16 == 0 && (uintptr_t)y % 16 == 0 && xbs % 16 == 0 && ybs % 16 == 0 &&
                      (!glu || n % 16 == 0)) ? 1 : 0;
  int64_t blocks = (n / 16 + 255) / 256;                   // one 16-byte access per thread ...
  const int64_t cap = (4096 + B - 1) / B;                  // ... up to about 16 workgroups per unit in all
  blocks = blocks < 1 ? 1 : (blocks > cap ? cap : blocks);
  if (B > 65535) return hipErrorInvalidValue;
  const dim3 grid((unsigned)blocks, (unsigned)B);
  if (glu) return launch_kernel(act_glu_kernel, grid, dim3(256), 0, st, c, x, y, n, xbs, ybs, vec_ok);
  return launch_kernel(act_unary_kernel, grid, dim3(256), 0, st, c, x, y, n, xbs, ybs, vec_ok);
}

hipError_t launch_softmax(const ActParams& c, const int32_t* x, int64_t rows, int32_t L, int8_t* y, hipStream_t st) {
  const unsigned grid = (unsigned)(rows < 8192 ? rows : 8192);
  return launch_kernel(softmax_kernel, dim3(grid), dim3(256), 0, st, c, x, rows, L, y);
}

}  // namespace qasr
