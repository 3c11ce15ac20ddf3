// The two steps either side of the integer path (paper Sec. 2.1): the quantiser of Eq. 1 with
// b = 8 that turns float32 features into int8 codes, and the dequantiser S * q that turns int8
// outputs back into float32.  Both are memory-bound elementwise passes (5 bytes per element):
// a thread handles 4 consecutive elements with one 16-byte and one 4-byte access when the
// pointers allow it, grid-stride over the tensor; the ragged ends go element by element.
//
// The arithmetic is fixed to single precision, step by step: clip to [-alpha, alpha], one
// correctly rounded division by S = alpha / 127 (S computed by the caller of the launch, on the
// host), round to nearest with ties to even; a NaN feature gives code 0.
#include "kernels.hpp"

namespace qasr {

namespace {

__device__ __forceinline__ int32_t quantize_one(float v, float alpha, float S) {
  if (v != v) return 0;
  v = v > alpha ? alpha : v;
  v = v < -alpha ? -alpha : v;
  return (int32_t)rintf(__fdiv_rn(v, S));
}

__global__ __launch_bounds__(256) void quantize_kernel(const float* __restrict__ x, size_t n, float alpha, float S,
                                                       int8_t* __restrict__ q, int vec_ok) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n4 = vec_ok ? n / 4 : 0;
  for (size_t i = tid; i < n4; i += stride) {
    const float4 v = reinterpret_cast<const float4*>(x)[i];
    const uint32_t pk = ((uint32_t)quantize_one(v.x, alpha, S) & 0xffu) | (((uint32_t)quantize_one(v.y, alpha, S) & 0xffu) << 8) |
                        (((uint32_t)quantize_one(v.z, alpha, S) & 0xffu) << 16) | ((uint32_t)quantize_one(v.w, alpha, S) << 24);
    reinterpret_cast<uint32_t*>(q)[i] = pk;
  }
  for (size_t i = 4 * n4 + tid; i < n; i += stride) q[i] = (int8_t)quantize_one(x[i], alpha, S);
}

__global__ __launch_bounds__(256) void dequantize_kernel(const int8_t* __restrict__ q, size_t n, float S,
                                                         float* __restrict__ x, int vec_ok) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n4 = vec_ok ? n / 4 : 0;
  for (size_t i = tid; i < n4; i += stride) {
    const uint32_t pk = reinterpret_cast<const uint32_t*>(q)[i];
    float4 v;
    v.x = __fmul_rn(S, (float)(int8_t)(pk & 0xffu));
    v.y = __fmul_rn(S, (float)(int8_t)((pk >> 8) & 0xffu));
    v.z = __fmul_rn(S, (float)(int8_t)((pk >> 16) & 0xffu));
    v.w = __fmul_rn(S, (float)(int8_t)(pk >> 24));
    reinterpret_cast<float4*>(x)[i] = v;
  }
  for (size_t i = 4 * n4 + tid; i < n; i += stride) x[i] = __fmul_rn(S, (float)q[i]);
}

unsigned grid_for(size_t n) {
  const size_t quads = (n + 3) / 4;
  const size_t blocks = (quads + 255) / 256;
  return (unsigned)(blocks < 1 ? 1 : (blocks > 4096 ? 4096 : blocks));   // >= 16 blocks per CU at full size
}

}  // namespace

hipError_t launch_quantize(const float* x, size_t n, float alpha, float S, int8_t* q, hipStream_t st) {
  const int vec_ok = ((uintptr_t)x % 16 == 0 && (uintptr_t)q % 4 == 0) ? 1 : 0;
  return launch_kernel(quantize_kernel, dim3(grid_for(n)), dim3(256), 0, st, x, n, alpha, S, q, vec_ok);
}

hipError_t launch_dequantize(const int8_t* q, size_t n, float S, float* x, hipStream_t st) {
  const int vec_ok = ((uintptr_t)x % 16 == 0 && (uintptr_t)q % 4 == 0) ? 1 : 0;
  return launch_kernel(dequantize_kernel, dim3(grid_for(n)), dim3(256), 0, st, q, n, S, x, vec_ok);
}

}  // namespace qasr
