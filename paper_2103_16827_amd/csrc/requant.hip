// Standalone layer epilogue on int32 accumulators: +bias, dyadic rescale, +residual, clamp.
// HBM-bound (4 B in, 1-2 B in/out per element): each thread turns 16 accumulators of one
// (b, c) row into 16 output bytes with 16-byte accesses when the row allows it.
#include "kernels.hpp"

namespace qasr {

__global__ __launch_bounds__(256) void requant_kernel(const int32_t* __restrict__ acc, int T,
                                                     int C, const int32_t* __restrict__ bias,
                                                     const int32_t* __restrict__ m,
                                                     const int32_t* __restrict__ s,
                                                     const int8_t* __restrict__ res, int relu,
                                                     int8_t* __restrict__ y, int vec_ok, int64_t row0) {
  const int64_t row = blockIdx.y;                 // (b * C + c) - row0; pointers are pre-offset
  const int c = (int)((row0 + row) % C);
  const int32_t bc = bias ? bias[c] : 0;
  const int32_t mc = m[c], sc = s[c];
  const int lo = relu ? 0 : -128;
  const int32_t* a = acc + row * T;
  const int8_t* r = res ? res + row * T : nullptr;
  int8_t* out = y + row * T;
  const int t0 = (blockIdx.x * blockDim.x + threadIdx.x) * 16;
  if (t0 >= T) return;
  if (vec_ok && t0 + 16 <= T) {
    int4 q[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) q[i] = *reinterpret_cast<const int4*>(a + t0 + 4 * i);
    int4 rr = make_int4(0, 0, 0, 0);
    if (r) rr = *reinterpret_cast<const int4*>(r + t0);
    const int32_t rw[4] = {rr.x, rr.y, rr.z, rr.w};
    int32_t ow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int32_t av[4] = {q[i].x, q[i].y, q[i].z, q[i].w};
      uint32_t pk = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int32_t v = dyadic_rescale(av[e] + bc, mc, sc);
        v += (int32_t)(int8_t)(rw[i] >> (8 * e));
        pk |= (uint32_t)(clamp_i8(v, lo) & 0xff) << (8 * e);
      }
      ow[i] = (int32_t)pk;
    }
    *reinterpret_cast<int4*>(out + t0) = make_int4(ow[0], ow[1], ow[2], ow[3]);
  } else {
    const int t1 = min(T, t0 + 16);
    for (int t = t0; t < t1; ++t) {
      int32_t v = dyadic_rescale(a[t] + bc, mc, sc);
      if (r) v += (int32_t)r[t];
      out[t] = (int8_t)clamp_i8(v, lo);
    }
  }
}

hipError_t launch_requant(const int32_t* acc, int B, int C, int T, const int32_t* bias,
                          const int32_t* m, const int32_t* s, const int8_t* res, int relu,
                          int8_t* y, hipStream_t st) {
  const int64_t rows = (int64_t)B * C;
  const int per_row = (T + 15) / 16;
  const int threads = per_row >= 256 ? 256 : (per_row > 64 ? 128 : 64);
  const int gx = (per_row + threads - 1) / threads;
  const int vec_ok = (T % 16 == 0) && ((uintptr_t)acc % 16 == 0) && ((uintptr_t)y % 16 == 0) &&
                     (!res || (uintptr_t)res % 16 == 0);
  for (int64_t r0 = 0; r0 < rows; r0 += 65535) {   // grid.y is limited to 65535 rows per launch
    const int64_t n = rows - r0 < 65535 ? rows - r0 : 65535;
    const hipError_t e = launch_kernel(requant_kernel, dim3(gx, (unsigned)n), dim3(threads), 0, st,
                                       acc + r0 * T, T, C, bias, m, s,
                                       res ? res + r0 * T : (const int8_t*)nullptr, relu,
                                       y + r0 * T, vec_ok, r0);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace qasr
