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
// Softmax: one wave per row up to 512 logits (no barrier, the row in registers), one workgroup per
// row beyond: extremes of the row, exponentials (kept in registers for rows up
// to 2048 logits, recomputed beyond) and their 64-bit sum, quotients.  The two divisions per
// element are 32-bit whenever the row's spread allows it (the choice is made per row and is
// wave-uniform): floor(-r / q_ln2) directly, and E 2^7 / sum through a 24-bit cut of both operands
// whose quotient the exact 64-bit remainder corrects by at most one.
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

// the table the elementwise kernel builds per workgroup, written out once (for layers whose
// epilogue applies the activation itself)
__global__ __launch_bounds__(256) void act_table_kernel(ActParams c, uint8_t* table) {
  const int q = (int)threadIdx.x - 128;
  const int32_t sg = sigmoid_code_dev(q, c);
  table[threadIdx.x] = (uint8_t)rescale_clamp(c.kind == 2 ? q * sg : sg, c.m, c.s);
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

// butterfly over the 64 lanes of a wave: every lane ends with the maximum / the sum
__device__ __forceinline__ long long wave_reduce(long long v, bool is_max) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const int lo = __shfl_xor((int)(uint32_t)(unsigned long long)v, o);
    const int hi = __shfl_xor((int)(uint32_t)((unsigned long long)v >> 32), o);
    const long long w = (long long)(((unsigned long long)(uint32_t)hi << 32) | (uint32_t)lo);
    v = is_max ? (w > v ? w : v) : v + w;
  }
  return v;
}

__device__ __forceinline__ long long wg_reduce(long long v, bool is_max, long long* sh) {
  // 256 threads: inside each wave first, then the four wave results through LDS
  v = wave_reduce(v, is_max);
  __syncthreads();                                   // sh may still be read from the previous use
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  const long long a = sh[0], b = sh[1], c = sh[2], d = sh[3];
  return is_max ? max(max(a, b), max(c, d)) : a + b + c + d;
}

// floor(n / d) for n < 2^31, 1 <= d < 2^30, when only quotients up to 63 matter (larger ones may come
// out as any value above 62): one multiplication by the reciprocal (single precision: the
// estimate is within one of the quotient while that is below 2^7), then the exact remainder
// decides.  rcp_d = 1.0f / (float)d.
__device__ __forceinline__ uint32_t div_small(uint32_t n, uint32_t d, float rcp_d, uint32_t& rem) {
  const float e = (float)n * rcp_d;
  uint32_t q = e >= 100.0f ? 100u : (uint32_t)e;               // only "> 62" matters up there
  int32_t r = (int32_t)(n - q * d);                             // q d <= 100 d and <= n (1 + 2^-22): no wrap that matters below 63
  if (q < 100u) {
    if (r < 0) { --q; r += (int32_t)d; }
    else if ((uint32_t)r >= d) { ++q; r -= (int32_t)d; }
  }
  rem = (uint32_t)r;
  return q;
}

// exp of r <= 0 when -r < 2^31 and q_ln2 < 2^30 (FAST, wave-uniform choice made per row), else the
// general form
template <bool FAST>
__device__ __forceinline__ long long iexp_row(long long r, const ActParams& c, float rcp_ql) {
  if (!FAST) return iexp_dev(r, c);
  const uint32_t nr = (uint32_t)(-r), ql = (uint32_t)c.q_ln2;
  uint32_t rem;
  const uint32_t z = div_small(nr, ql, rcp_ql, rem);
  const long long tp = (long long)((int32_t)(uint32_t)c.q_b - (int32_t)rem);      // p + q_b, p = -rem
  const long long L = tp * tp + c.q_c;
  return z > 62 ? 0 : (L >> z);
}

// floor(a / b) for 0 <= a <= 128 b, 1 <= b < 2^55: both operands are cut to b's leading 24 bits
// (shift sh, b1 = b >> sh, rcp_b1 = 1.0f / (float)b1); the single-precision quotient of the cuts is
// within one of the true one (the cuts move a/b by less than 2^-15, the arithmetic by less than
// 2^-14), and the exact 64-bit remainder decides.
__device__ __forceinline__ uint32_t div_small_quotient(unsigned long long a, unsigned long long b, int sh, float rcp_b1) {
  const uint32_t a1 = (uint32_t)(a >> sh);
  uint32_t q = (uint32_t)((float)a1 * rcp_b1);
  const long long rem = (long long)a - (long long)((unsigned long long)q * b);
  if (rem < 0) --q;
  else if ((unsigned long long)rem >= b) ++q;
  return q;
}

template <bool FAST>
__device__ __forceinline__ void softmax_row(const ActParams& c, const int32_t* __restrict__ xr, int32_t L,
                                            int8_t* __restrict__ yr, long long mx, long long* sh) {
  constexpr int K = 8;                               // elements per thread kept in registers
  const long long mul = 1ll << c.u;
  const float rcp_ql = 1.0f / (float)(uint32_t)(c.q_ln2 < (1ll << 30) ? c.q_ln2 : 1);
  if (L <= 256 * K) {
    long long E[K];
    long long sum = 0;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int j = threadIdx.x + 256 * k;
      E[k] = j < L ? iexp_row<FAST>(((long long)xr[j] - mx) * mul, c, rcp_ql) : 0;
      sum += E[k];
    }
    sum = wg_reduce(sum, false, sh);
    const int shn = max(0, 40 - __clzll(sum));       // sum >> shn has at most 24 bits
    const float rcp_b1 = 1.0f / (float)(uint32_t)((unsigned long long)sum >> shn);
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int j = threadIdx.x + 256 * k;
      if (j < L) {
        const uint32_t p = div_small_quotient((unsigned long long)E[k] << 7, (unsigned long long)sum, shn, rcp_b1);
        yr[j] = (int8_t)(p > 127 ? 127 : p);
      }
    }
  } else {
    long long sum = 0;
    for (int j = threadIdx.x; j < L; j += 256) sum += iexp_row<FAST>(((long long)xr[j] - mx) * mul, c, rcp_ql);
    sum = wg_reduce(sum, false, sh);
    const int shn = max(0, 40 - __clzll(sum));
    const float rcp_b1 = 1.0f / (float)(uint32_t)((unsigned long long)sum >> shn);
    for (int j = threadIdx.x; j < L; j += 256) {
      const unsigned long long E = (unsigned long long)iexp_row<FAST>(((long long)xr[j] - mx) * mul, c, rcp_ql);
      const uint32_t p = div_small_quotient(E << 7, (unsigned long long)sum, shn, rcp_b1);
      yr[j] = (int8_t)(p > 127 ? 127 : p);
    }
  }
}

__global__ __launch_bounds__(256) void softmax_kernel(ActParams c, const int32_t* __restrict__ x, int64_t rows, int32_t L,
                                                      int8_t* __restrict__ y) {
  __shared__ long long sh[4];
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
    const int32_t* xr = x + row * L;
    int8_t* yr = y + row * L;
    long long mx = INT32_MIN, mn = INT32_MAX;
    for (int j = threadIdx.x; j < L; j += 256) {
      const long long v = xr[j];
      mx = max(mx, v);
      mn = min(mn, v);
    }
    mx = wg_reduce(mx, true, sh);
    mn = -wg_reduce(-mn, true, sh);
    // every (max - q) 2^u of the row below 2^31, and the constants too: 32-bit exponentials
    const bool fast = ((mx - mn) << c.u) < (1ll << 31) && c.q_ln2 < (1ll << 30);
    if (fast) softmax_row<true>(c, xr, L, yr, mx, sh);
    else softmax_row<false>(c, xr, L, yr, mx, sh);
  }
}

// Rows of up to 512 logits: one wave per row (no barrier, the row lives in registers: 8 logits per
// lane), four rows per workgroup.
template <bool FAST>
__device__ __forceinline__ void softmax_wave_row(const ActParams& c, const int32_t (&xv)[8], int32_t L, int lane,
                                                 int8_t* __restrict__ yr, long long mx) {
  const long long mul = 1ll << c.u;
  const float rcp_ql = 1.0f / (float)(uint32_t)(c.q_ln2 < (1ll << 30) ? c.q_ln2 : 1);
  long long E[8];
  long long sum = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    E[k] = lane + 64 * k < L ? iexp_row<FAST>(((long long)xv[k] - mx) * mul, c, rcp_ql) : 0;
    sum += E[k];
  }
  sum = wave_reduce(sum, false);
  const int shn = max(0, 40 - __clzll(sum));
  const float rcp_b1 = 1.0f / (float)(uint32_t)((unsigned long long)sum >> shn);
#pragma unroll
  for (int k = 0; k < 8; ++k)
    if (lane + 64 * k < L) {
      const uint32_t p = div_small_quotient((unsigned long long)E[k] << 7, (unsigned long long)sum, shn, rcp_b1);
      yr[lane + 64 * k] = (int8_t)(p > 127 ? 127 : p);
    }
}

__global__ __launch_bounds__(256) void softmax_wave_kernel(ActParams c, const int32_t* __restrict__ x, int64_t rows,
                                                           int32_t L, int8_t* __restrict__ y) {
  const int lane = threadIdx.x & 63;
  const int64_t nw = (int64_t)gridDim.x * 4;
  auto load_row = [&](int64_t row, int32_t (&v)[8]) {
    const int32_t* xr = x + row * L;
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = lane + 64 * k < L ? xr[lane + 64 * k] : 0;
  };
  int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  int32_t xv[8], xn[8];
  load_row(row, xv);
  for (; row < rows; row += nw) {
    const bool more = row + nw < rows;               // the next row of this wave is on its way while this one is worked on
    if (more) load_row(row + nw, xn);
    long long mx = INT32_MIN, mn = INT32_MAX;
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (lane + 64 * k < L) {
        mx = max(mx, (long long)xv[k]);
        mn = min(mn, (long long)xv[k]);
      }
    mx = wave_reduce(mx, true);
    mn = -wave_reduce(-mn, true);
    const bool fast = ((mx - mn) << c.u) < (1ll << 31) && c.q_ln2 < (1ll << 30);      // wave-uniform
    if (fast) softmax_wave_row<true>(c, xv, L, lane, y + row * L, mx);
    else softmax_wave_row<false>(c, xv, L, lane, y + row * L, mx);
    if (more) {
#pragma unroll
      for (int k = 0; k < 8; ++k) xv[k] = xn[k];
    }
  }
}

}  // namespace

hipError_t launch_act_table(const ActParams& c, uint8_t* table, hipStream_t st) {
  hipLaunchKernelGGL(act_table_kernel, dim3(1), dim3(256), 0, st, c, table);
  return hipGetLastError();
}

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
  if (L <= 512) {
    const int64_t wgs = (rows + 3) / 4;
    return launch_kernel(softmax_wave_kernel, dim3((unsigned)(wgs < 2048 ? wgs : 2048)), dim3(256), 0, st, c, x, rows, L, y);
  }
  const unsigned grid = (unsigned)(rows < 8192 ? rows : 8192);
  return launch_kernel(softmax_kernel, dim3(grid), dim3(256), 0, st, c, x, rows, L, y);
}

}  // namespace qasr
