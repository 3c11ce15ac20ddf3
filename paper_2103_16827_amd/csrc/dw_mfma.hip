// Depthwise int8 convolution (stride 1) on the gfx950 int8 matrix cores, with the fused
// epilogue (bias, dyadic rescale, residual, clamp).
//
// A depthwise layer moves 2 bytes per output but needs k = 33..87 multiply-adds for it, which
// is beyond what the vector ALUs sustain at HBM speed.  The per-channel convolution is
// therefore written as a product with a banded Toeplitz matrix and issued on MFMA:
//
//     Y[m, n] = sum_kappa A[m, kappa] * X[kappa, n]        (v_mfma_i32_16x16x64_i8)
//     output frame   t = T0 + 16 n + m                      (n: 16-frame group, m: frame in group)
//     X[kappa, n]    = x[o + 16 n + kappa],   o = T0 - pad_left - delta   (o is a multiple of 16)
//     A[m, kappa]    = w[j]  if kappa - m - delta == j * dilation, else 0
//
// so a lane's 16-byte X operand is 16 consecutive frames at a 16-byte aligned position, and the
// matrix-core time is negligible next to the memory time.  One workgroup = one channel (one A
// operand, built once and shared through LDS) x 4 waves; a wave owns R "strips" (a batch item's
// row, or a 1024-frame segment of it), stages them in LDS with their zero halos, and walks the
// 16-frame groups of all its strips as one flat column space so that MFMA tiles stay full
// across row ends.
#include "kernels.hpp"
#include "tuning.hpp"

#include <cstdlib>
#include <type_traits>

namespace qasr {

typedef int v4i __attribute__((ext_vector_type(4)));

namespace {

constexpr int kSeg = 1024;   // output frames per strip when a row is longer than this

struct DwGeom {
  int delta;     // (-pad_left) mod 16
  int PH;        // (pad_left + delta) / 16: left halo in 16-byte chunks
  int nseg;      // strips per row
  int R;         // strips per wave
  int NI;        // 64-lane load rounds per strip
  int NCH;       // 16-byte chunks per strip buffer: groups + 4*KC - 1
  int nstrips;   // B * nseg
  int aligned_out;
  int c_per_xcd; // channels per XCD: ceil(C / 8)
};

template <int KC, bool ALIGNED>
__global__ __launch_bounds__(256) void dw_mfma_kernel(ConvParams p, DwGeom g) {
  extern __shared__ __align__(16) unsigned char strips_lds[];      // [4 waves][R][NCH][16]
  __shared__ __align__(16) unsigned char a_lds[KC * 1024];         // A operand, register layout
  __shared__ unsigned char wrow[64 * KC + 16];                     // dilated, shifted weight row

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // Consecutive workgroups go round-robin to the 8 XCDs (one L2 each); rows of neighbouring
  // channels share a cache line where they meet, so each XCD takes a contiguous range of channels.
  const int c = (int)(blockIdx.x & 7) * g.c_per_xcd + (int)(blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= g.c_per_xcd || c >= p.Cout) return;   // whole workgroup
  const int n = lane & 15, gi = lane >> 4;
  const int strip0 = (blockIdx.y * 4 + wave) * g.R;
  const int Rv = min(g.R, g.nstrips - strip0);                     // <= 0: this wave has no work
  unsigned char* my = strips_lds + (size_t)wave * g.R * g.NCH * 16;

  // ---- 1. start the global loads of this wave's strips (chunk u of strip r -> lane u % 64)
  int4 xv[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    xv[i] = make_int4(0, 0, 0, 0);
    if (i < g.R * g.NI) {
      const int r = g.NI == 2 ? (i >> 1) : i;
      const int u = lane + 64 * (g.NI == 2 ? (i & 1) : 0);
      if (r < Rv && u < g.NCH) {
        const int strip = strip0 + r;
        const int b = strip / g.nseg;
        const int T0 = (strip - b * g.nseg) * kSeg;
        const int t = T0 + 16 * (u - g.PH);                        // first frame of the chunk
        const int8_t* row = p.x + (int64_t)b * p.xbs + (int64_t)c * p.Tin;
        if (ALIGNED) {
          if (t >= 0 && t < p.Tin) xv[i] = *reinterpret_cast<const int4*>(row + t);
        } else if (t > -16 && t < p.Tin) {
          uint32_t d[4] = {0, 0, 0, 0};
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int tt = t + e;
            if (tt >= 0 && tt < p.Tin) d[e >> 2] |= (uint32_t)(uint8_t)row[tt] << (8 * (e & 3));
          }
          xv[i] = make_int4((int)d[0], (int)d[1], (int)d[2], (int)d[3]);
        }
      }
    }
  }

  // per-channel constants: uniform over the workgroup, requested before anything waits
  const int32_t bias = p.bias ? p.bias[c] : 0;
  const int32_t mc = p.m[c], sc = p.s[c];

  // ---- 2. Toeplitz operand: wrow[q] = w[j] where q - 15 - delta == j * dilation
  for (int q = tid; q < 64 * KC + 16; q += 256) {
    const int rel = q - 15 - g.delta;
    int8_t v = 0;
    if (rel >= 0) {
      const int j = rel / p.dil;
      if (j * p.dil == rel && j < p.k) v = p.w[(int64_t)c * p.k + j];
    }
    wrow[q] = (unsigned char)v;
  }
  __syncthreads();
  {
    // A[m, kappa] = wrow[kappa - m + 15]; lane (m, gi) holds kappa = 64 kc + 16 gi + (0..15).
    const int al = tid >> 2, dwi = tid & 3;
    const int am = al & 15, ag = al >> 4;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const int base = 64 * kc + 16 * ag + 4 * dwi - am + 15;
      const uint32_t v = (uint32_t)wrow[base] | ((uint32_t)wrow[base + 1] << 8) |
                         ((uint32_t)wrow[base + 2] << 16) | ((uint32_t)wrow[base + 3] << 24);
      reinterpret_cast<uint32_t*>(a_lds)[kc * 256 + tid] = v;
    }
  }

  // ---- 3. strips (with their zero halos) to LDS
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (i < g.R * g.NI) {
      const int r = g.NI == 2 ? (i >> 1) : i;
      const int u = lane + 64 * (g.NI == 2 ? (i & 1) : 0);
      if (u < g.NCH) *reinterpret_cast<int4*>(my + ((size_t)r * g.NCH + u) * 16) = xv[i];
    }
  }
  __syncthreads();
  if (Rv <= 0) return;

  v4i a[KC];
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) a[kc] = *reinterpret_cast<const v4i*>(a_lds + kc * 1024 + lane * 16);

  // groups per strip: all strips of a wave have the same count (R > 1 only when nseg == 1)
  const int b0 = strip0 / g.nseg;
  const int T0w = (strip0 - b0 * g.nseg) * kSeg;
  const int G = (min(kSeg, p.Tout - T0w) + 15) >> 4;
  const int ntiles = (Rv * G + 15) >> 4;
  const int lo = p.relu ? 0 : -128;

  // Output addressing: wave-uniform 64-bit base + a 32-bit per-lane offset.  Strip r of the wave is
  // batch item b0 + r (nseg == 1) or the only strip (R == 1); the host keeps R * ybs below 2^31.
  const int64_t obase = (int64_t)b0 * p.ybs + (int64_t)c * p.Tout + T0w;
  int8_t* const yb = p.y + obase;
  const int8_t* const rb = p.res ? p.res + obase : nullptr;
  const int strip_pitch = g.nseg == 1 ? (int)p.ybs : 0;
  const int Tleft = p.Tout - T0w;                     // frames of this strip from its first frame

  // column walk: lane n starts at column n of strip 0 and advances 16 columns per tile
  int r = 0, grp = n;
  while (grp >= G) { grp -= G; ++r; }

  auto tile_loop = [&](auto fast_tag) {
    constexpr bool FAST = decltype(fast_tag)::value;
    const int sh = FAST ? sc - 32 : 0;
    const int rnd = FAST ? 1 << (sc - 33) : 0;
    for (int tile = 0; tile < ntiles; ++tile) {
      const bool valid = r < Rv;
      const int rr_ = valid ? r : 0;
      const unsigned char* bp = my + ((rr_ * g.NCH + grp + gi) << 4);
      v4i acc = {bias, bias, bias, bias};
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        const v4i xb = *reinterpret_cast<const v4i*>(bp + kc * 64);
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[kc], xb, acc, 0, 0, 0);
      }
      const int t = 16 * grp + 4 * gi;                // frame inside the strip
      if (valid && t < Tleft) {
        const int o = rr_ * strip_pitch + t;
        int32_t v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
          v[i] = FAST ? ((int32_t)__mulhi(acc[i], mc) + rnd) >> sh : dyadic_rescale(acc[i], mc, sc);
        if (g.aligned_out) {
          if (rb) {
            const uint32_t rw = *reinterpret_cast<const uint32_t*>(rb + o);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] += (int32_t)(int8_t)(rw >> (8 * i));
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = clamp_i8(v[i], lo);
          const uint32_t p01 = __builtin_amdgcn_perm((uint32_t)v[1], (uint32_t)v[0], 0x0c0c0400u);
          const uint32_t p23 = __builtin_amdgcn_perm((uint32_t)v[3], (uint32_t)v[2], 0x04000c0cu);
          *reinterpret_cast<uint32_t*>(yb + o) = p01 | p23;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if (t + i < Tleft) {
              int32_t w_ = v[i];
              if (rb) w_ += (int32_t)rb[o + i];
              yb[o + i] = (int8_t)clamp_i8(w_, lo);
            }
          }
        }
      }
      grp += 16;
      while (grp >= G) { grp -= G; ++r; }
    }
  };
  if (sc >= 33) tile_loop(std::true_type{}); else tile_loop(std::false_type{});
}

bool geometry(const ConvParams& p, DwGeom& g, int& KC) {
  if (!p.depthwise || p.stride != 1 || p.Tout < 1) return false;
  g.delta = ((-p.pl) % 16 + 16) % 16;
  g.PH = (p.pl + g.delta) / 16;
  const int64_t need = 16 + g.delta + (int64_t)p.dil * (p.k - 1);
  if (need > 256) return false;
  KC = (int)((need + 63) / 64);
  g.nseg = (p.Tout + kSeg - 1) / kSeg;
  const int Gfull = g.nseg > 1 ? kSeg / 16 : (p.Tout + 15) / 16;
  g.NCH = Gfull + 4 * KC - 1;
  g.NI = (g.NCH + 63) / 64;
  const int64_t nstrips = (int64_t)p.B * g.nseg;
  if (nstrips > 0x3fffffff) return false;
  g.nstrips = (int)nstrips;
  // strips per wave: keep MFMA tiles full across row ends without starving the chip of workgroups
  g.R = 1;
  if (g.nseg == 1) {
    double best = -1.0;
    for (int R = 1; R <= 8 / g.NI && R <= p.B && (int64_t)R * p.ybs < 0x7fffffffLL; R *= 2) {
      const int cols = R * Gfull;
      const double eff = (double)cols / (16.0 * ((cols + 15) / 16));
      const double blocks = (double)p.Cout * ((p.B + 4 * R - 1) / (4 * R));
      const double fill = blocks >= 1024.0 ? 1.0 : blocks / 1024.0;
      const double score = eff * (0.25 + 0.75 * fill);
      if (score > best + 1e-9) { best = score; g.R = R; }
    }
  }
  {                                                      // tuning override: strips per wave
    const int R = tuning().dw_r;
    if (g.nseg == 1 && (R == 1 || R == 2 || R == 4 || R == 8) && R * g.NI <= 8 &&
        (int64_t)R * p.ybs < 0x7fffffffLL)
      g.R = R;
  }
  const int64_t gy = (nstrips + 4 * g.R - 1) / (4 * g.R);
  if (gy > 65535) return false;
  g.c_per_xcd = (p.Cout + 7) / 8;
  g.aligned_out = (p.Tout % 4 == 0) && ((uintptr_t)p.y % 4 == 0) && (p.ybs % 4 == 0) &&
                  (!p.res || (uintptr_t)p.res % 4 == 0);
  return true;
}

template <int KC>
hipError_t launch_kc(const ConvParams& p, const DwGeom& g, hipStream_t st) {
  const dim3 grid(8 * g.c_per_xcd, (g.nstrips + 4 * g.R - 1) / (4 * g.R));
  const size_t shmem = (size_t)4 * g.R * g.NCH * 16;
  const bool aligned = (p.Tin % 16 == 0) && ((uintptr_t)p.x % 16 == 0) && (p.xbs % 16 == 0);
  if (aligned) return launch_kernel(dw_mfma_kernel<KC, true>, grid, dim3(256), shmem, st, p, g);
  return launch_kernel(dw_mfma_kernel<KC, false>, grid, dim3(256), shmem, st, p, g);
}

}  // namespace

bool dw_mfma_supported(const ConvParams& p) {
  DwGeom g;
  int KC;
  return geometry(p, g, KC);
}

hipError_t launch_dw_mfma(const ConvParams& p, hipStream_t st) {
  DwGeom g;
  int KC;
  if (!geometry(p, g, KC)) return hipErrorInvalidValue;
  switch (KC) {
    case 1: return launch_kc<1>(p, g, st);
    case 2: return launch_kc<2>(p, g, st);
    case 3: return launch_kc<3>(p, g, st);
    default: return launch_kc<4>(p, g, st);
  }
}

}  // namespace qasr
