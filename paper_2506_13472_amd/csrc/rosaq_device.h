// Small device helpers shared by the kernel files.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace rosaq {

// fp64 -> fp16 with a single round-half-to-even step: scale so that the fp16 ulp is 1
// (exact power-of-two scaling), round to integer, reassemble the bit pattern.
__device__ __forceinline__ uint16_t f64_to_f16_bits(double v) {
  const uint16_t sign = v < 0.0 || (v == 0.0 && __builtin_signbit(v)) ? 0x8000u : 0u;
  if (v != v) return 0x7e00u;
  const double a = __builtin_fabs(v);
  if (a >= 65520.0) return sign | 0x7c00u;
  if (a < 6.103515625e-05) {                      // below 2^-14: subnormal grid, ulp 2^-24
    return sign | static_cast<uint16_t>(__builtin_rint(__builtin_ldexp(a, 24)));
  }
  int e;
  (void)__builtin_frexp(a, &e);                   // a = f * 2^e, f in [0.5, 1)
  e -= 1;
  double m = __builtin_rint(__builtin_ldexp(a, 10 - e));   // in [1024, 2048]
  if (m >= 2048.0) { m = 1024.0; e += 1; }
  return sign | static_cast<uint16_t>(((e + 15) << 10) + (static_cast<int>(m) - 1024));
}

__device__ __forceinline__ double f16_bits_to_f64(uint16_t h) {
  return static_cast<double>(__builtin_bit_cast(_Float16, h));   // exact
}

}  // namespace rosaq
