// Shared device helpers and launch-parameter structs of the HIP path (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace qasr {

// Geometry + pointers of one layer, passed by value to every convolution kernel.
struct ConvParams {
  const int8_t* x;
  const int8_t* w;
  const int32_t* bias;   // may be null
  const int32_t* m;
  const int32_t* s;
  const int8_t* res;     // may be null
  int8_t* y;
  int64_t xbs, ybs;      // batch strides in elements
  int32_t B, Cin, Cout, Tin, Tout;
  int32_t k, stride, dil, pl;
  int32_t depthwise;     // 0: groups == 1, 1: groups == Cin == Cout
  int32_t relu;
  int32_t w_packed;      // groups == 1, Cin % 64 == 0: weights are in MFMA operand order (below)
  // dense-residual layers: further residual operands (same shape and stride as `res`), all added
  // to the rescaled value before the one clamp; only conv_pipe and conv_generic read them
  int32_t n_res_more;
  const int8_t* res_more[11];
  // unary activation fused into the epilogue: 256 bytes, entry (code + 128) = the activation's int8
  // output for that int8 code (built once by act_table_kernel); null = none.  Only pw_pipe and dw_pipe read it.
  const uint8_t* act_lut;
};
constexpr int kMaxMoreRes = 11;

// Packed weight layout (groups == 1, Cin % 64 == 0): [k][ceil(Cout/16)][Cin/64][64 lanes][16 bytes].
// Lane l = 16*gi + n of block (j, co16, kc) holds output channel co = 16*co16 + n (zeros beyond
// Cout) and, in its bytes e = 0..15, the input channels
//     ci = 64*kc + 8*gi + e            (e < 8)
//     ci = 64*kc + 32 + 8*gi + (e - 8) (e >= 8)
// which is the order in which the activation operand of the matrix-core kernels is assembled.
// One wave-wide 16-byte load of a block is 1 KiB of contiguous memory.
__host__ __device__ inline int64_t packed_weight_index(int j, int co, int ci, int Cout, int Cin) {
  const int co16n = (Cout + 15) >> 4, kch = Cin >> 6;
  const int kc = ci >> 6, r = ci & 63;
  const int gi = (r & 31) >> 3, e = (r & 7) + ((r >> 5) << 3);
  const int lane = gi * 16 + (co & 15);
  return ((((int64_t)j * co16n + (co >> 4)) * kch + kc) * 64 + lane) * 16 + e;
}

// Dyadic rescale v = floor((A*m + 2^(s-1)) / 2^s), 0 <= m < 2^31, 1 <= s <= 62, returned
// clamped to [-2^20, 2^20] (the caller adds an int8 residual and clamps to int8 next, so any
// value beyond +-256 is equivalent).
//
// For s >= 33 write A*m = H*2^32 + L with 0 <= L < 2^32 and H = mulhi(A, m).  Then
// floor((A*m + 2^(s-1)) / 2^s) = floor((H + 2^(s-33) + L/2^32) / 2^(s-32)); the numerator's
// integer part has a fractional remainder of at most 1 - 2^-(s-32) after division and
// L/2^s < 2^-(s-32) cannot carry, so the result is (H + 2^(s-33)) >> (s-32): one high
// multiply, one add, one arithmetic shift.  Smaller s takes the 64-bit form.
__device__ __forceinline__ int32_t dyadic_rescale(int32_t A, int32_t m, int32_t s) {
  if (s >= 33) {
    const int32_t h = __mulhi(A, m);
    return (h + (1 << (s - 33))) >> (s - 32);
  }
  long long v = ((long long)A * (long long)m + (1ll << (s - 1))) >> s;
  v = v > (1 << 20) ? (1 << 20) : v;
  v = v < -(1 << 20) ? -(1 << 20) : v;
  return (int32_t)v;
}

// The same rescale in its 64-bit form only (any 1 <= s <= 62), clamped like dyadic_rescale.
__device__ __forceinline__ int32_t dyadic_rescale64(int32_t A, int32_t m, int32_t s) {
  long long v = ((long long)A * (long long)m + (1ll << (s - 1))) >> s;
  v = v > (1 << 20) ? (1 << 20) : v;
  v = v < -(1 << 20) ? -(1 << 20) : v;
  return (int32_t)v;
}

// Launch through hipLaunchKernel so that the status returned is this launch's own (the
// thread-wide "last error" may hold a stale, unrelated value left by other HIP users).
// Arguments are converted to the kernel's own parameter types before their addresses are taken.
template <typename T> struct same_type { using type = T; };
template <typename... KArgs>
inline hipError_t launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t shmem,
                                hipStream_t st, typename same_type<KArgs>::type... args) {
  void* argv[] = {(void*)&args...};
  return hipLaunchKernel((const void*)kernel, grid, block, argv, shmem, st);
}

// Raises a kernel's dynamic-LDS limit (to the chip's 160 KiB unless the kernel also has static LDS
// and says how much dynamic LDS it needs) once per device: `done` (one per kernel
// instantiation) holds a bit per device ordinal; two threads racing here both set the attribute,
// which is harmless.  Devices beyond the mask's width set it on every launch.
inline hipError_t ensure_max_dynamic_lds(const void* kernel, std::atomic<uint64_t>& done, int bytes = 160 * 1024) {
  int dev = 0;
  const hipError_t ge = hipGetDevice(&dev);
  if (ge != hipSuccess) return ge;
  const uint64_t bit = (dev >= 0 && dev < 64) ? (uint64_t)1 << dev : 0;
  if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
  return e;
}

__device__ __forceinline__ int32_t clamp_i8(int32_t v, int32_t lo) {
  return min(127, max(lo, v));
}

// high 32 bits of the signed 64-bit product, in one instruction whatever the surrounding code
// looks like (the compiler only forms it when both sign extensions sit in the same basic block;
// with one of them hoisted out of a loop it expands a 64 x 64 multiply instead)
__device__ __forceinline__ int32_t mulhi_i32(int32_t a, int32_t b) {
  int32_t r;
  asm("v_mul_hi_i32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// median of three = clamp(x, lo, hi) for lo <= hi, in one instruction (the compiler only forms it
// by itself when both bounds are compile-time constants)
__device__ __forceinline__ int32_t med3_i32(int32_t x, int32_t lo, int32_t hi) {
  int32_t r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(lo), "v"(hi));
  return r;
}

// Epilogue of 4 accumulators of one channel (4 consecutive frames): dyadic rescale, residual bytes
// of `resw` added (pass 0 for none), clamp to [lo, 127], packed little-endian into one dword.
// FAST: s >= 33, sh = s - 32, rnd = 2^(s-33) (see dyadic_rescale); otherwise sh carries s itself.
template <bool FAST, bool RES>
__device__ __forceinline__ uint32_t requant_pack4(const int32_t (&a)[4], int32_t m, int32_t sh, int32_t rnd,
                                                  uint32_t resw, int32_t lo, int32_t hi127) {
  int32_t v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[i] = FAST ? ((int32_t)__mulhi(a[i], m) + rnd) >> sh : dyadic_rescale64(a[i], m, sh);
    if (RES) v[i] += (int32_t)(int8_t)(resw >> (8 * i));
    v[i] = med3_i32(v[i], lo, hi127);
  }
  const uint32_t p01 = __builtin_amdgcn_perm((uint32_t)v[1], (uint32_t)v[0], 0x0c0c0400u);
  const uint32_t p23 = __builtin_amdgcn_perm((uint32_t)v[3], (uint32_t)v[2], 0x04000c0cu);
  return p01 | p23;
}

}  // namespace qasr
