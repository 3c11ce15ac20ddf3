// Two measured ceilings of the chip this library runs on, for benchmarks that want to quote a
// kernel against what the machine does rather than against the datasheet:
//   * a streaming int8 copy (16 bytes per lane and step, every workgroup a contiguous share), the
//     rate HBM sustains for a read plus a write of the same size;
//   * a register-resident loop of v_mfma_i32_16x16x64_i8 (no memory traffic at all, independent
//     accumulators), the rate at which the matrix cores retire int8 products.
// Neither is part of the inference path.
#include "kernels.hpp"

namespace qasr {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kCopyThreads = 256;
constexpr int kMfmaThreads = 256;   // four waves, one per SIMD
constexpr int kMfmaAcc = 8;         // independent accumulators per wave

__global__ __launch_bounds__(kCopyThreads) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                                  size_t n16) {
  // workgroup g takes the g-th contiguous share, four 16-byte elements per lane in flight
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = per * blockIdx.x;
  const size_t hi = lo + per < n16 ? lo + per : n16;
  size_t i = lo + threadIdx.x;
  for (; i + 3 * kCopyThreads < hi; i += 4 * kCopyThreads) {
    const uint4 a = src[i], b = src[i + kCopyThreads], c = src[i + 2 * kCopyThreads], d = src[i + 3 * kCopyThreads];
    dst[i] = a;
    dst[i + kCopyThreads] = b;
    dst[i + 2 * kCopyThreads] = c;
    dst[i + 3 * kCopyThreads] = d;
  }
  for (; i < hi; i += kCopyThreads) dst[i] = src[i];
}

__global__ __launch_bounds__(kMfmaThreads) void probe_mfma_kernel(int iters, int32_t* __restrict__ out) {
  v4i a, b;
  const int t = threadIdx.x;
  a = v4i{t, t + 1, t + 2, t + 3};
  b = v4i{3 * t, 5 * t, 7 * t, 11 * t};
  v4i acc[kMfmaAcc];
#pragma unroll
  for (int j = 0; j < kMfmaAcc; ++j) acc[j] = v4i{j, 0, 0, 0};
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int j = 0; j < kMfmaAcc; ++j) acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[j], 0, 0, 0);
  }
  v4i s = acc[0];
#pragma unroll
  for (int j = 1; j < kMfmaAcc; ++j) s += acc[j];
  // one value per workgroup keeps the loop alive; the stores are a few hundred bytes in all
  if (t == 0) out[blockIdx.x] = s[0] + s[1] + s[2] + s[3];
}

}  // namespace

hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  const size_t want = (n16 + 4 * kCopyThreads - 1) / (4 * kCopyThreads);
  const unsigned grid = (unsigned)(want < 256 * 16 ? want : 256 * 16);
  hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(kCopyThreads), 0, st, (const uint4*)src, (uint4*)dst, n16);
  return hipGetLastError();
}

int probe_mfma_workgroups() { return 256 * 8; }   // eight workgroups of four waves per compute unit

double probe_mfma_ops(int iters) {
  // one instruction is a 16x16 tile over a contraction of 64: 16384 multiply-adds
  return 2.0 * 16384.0 * kMfmaAcc * (double)iters * (kMfmaThreads / 64) * probe_mfma_workgroups();
}

hipError_t launch_probe_mfma(int iters, int32_t* out, hipStream_t st) {
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(probe_mfma_workgroups()), dim3(kMfmaThreads), 0, st, iters, out);
  return hipGetLastError();
}

}  // namespace qasr
