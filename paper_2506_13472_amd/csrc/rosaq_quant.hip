// Offline step on the GPU (Sec. 3.2-3.3, Eq. 3): from the rotated weight What16 = fp16(W Q),
// already in device memory, to the packed layer in one pass -- the fp16 salient block, per
// (output row, group) min / max, scale, zero point and codes -- written straight into the
// fragment-ordered images the run-time kernels read, plus the layout-independent arrays that
// rosaq_packed_export returns.  Scale and zero point are computed in fp64 exactly as the host
// packer does (the quotients lie far enough from every rounding boundary for fp64, not for
// fp32), so the result is bit-identical to the host path.
#include <hip/hip_runtime.h>

#include <string>

#include "rosaq_device.h"
#include "rosaq_internal.h"

namespace rosaq {

// One wave per (16-channel tile, group) record.  Lane l owns output row 16 tile + l % 16 and, for
// each of the group's four k-steps t, the eight storage columns 128 g + 32 t + 8 (l / 16) + e:
// exactly the 32 codes of its 16-byte (INT4) or 12-byte (INT3) slot in the record.
template <int BITS>
__global__ __launch_bounds__(256) void quantize_pack_kernel(
    const uint16_t* __restrict__ what, int N, int D, int K, int G, int ntiles,
    const int32_t* __restrict__ perm, uint32_t* __restrict__ wq, uint8_t* __restrict__ codes,
    uint16_t* __restrict__ scales, uint16_t* __restrict__ zeros, unsigned* __restrict__ flag) {
  constexpr int kCodeDwords = BITS == 4 ? 256 : 192, kRecDwords = kCodeDwords + 16;
  const int lane = threadIdx.x & 63;
  const int rec = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (rec >= ntiles * G) return;
  const int tile = rec / G, g = rec - tile * G;
  const int r = lane & 15, kq = lane >> 4;
  const int n = tile * kTileN + r;
  const bool valid = n < N;
  const int C = D - K;

  double w[32];
  double mn = INFINITY, mx = -INFINITY;
  bool bad = false;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int p = K + g * kGroup + t * kKStep + kq * 8 + e;
      const uint16_t h = valid ? what[static_cast<size_t>(n) * D + perm[p]] : uint16_t{0};
      bad |= ((h >> 10) & 31) == 31;
      const double v = f16_bits_to_f64(h);
      w[t * 8 + e] = v;
      mn = fmin(mn, v);
      mx = fmax(mx, v);
    }
  // the four lanes of a row (l % 16 equal) hold a quarter of the group each
  mn = fmin(mn, __shfl_xor(mn, 16, 64)); mn = fmin(mn, __shfl_xor(mn, 32, 64));
  mx = fmax(mx, __shfl_xor(mx, 16, 64)); mx = fmax(mx, __shfl_xor(mx, 32, 64));
  if (bad) atomicOr(flag, 1u);

  const double qmax = static_cast<double>((1 << BITS) - 1);
  const uint16_t s16 = f64_to_f16_bits(fmax((mx - mn) / qmax, 6.103515625e-05));
  const double s = f16_bits_to_f64(s16);
  const double z = fmin(fmax(__builtin_rint(-mn / s), 0.0), qmax);
  uint32_t q[32];
#pragma unroll
  for (int i = 0; i < 32; ++i)
    q[i] = static_cast<uint32_t>(fmin(fmax(__builtin_rint(w[i] / s) + z, 0.0), qmax));

  uint32_t* record = wq + static_cast<size_t>(rec) * kRecDwords;
  if (BITS == 4) {
    // dword t holds k-step t; element e sits in nibble (e >> 1) + 4 (e & 1)
    uint32_t v[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      v[t] = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) v[t] |= q[t * 8 + e] << (4 * ((e >> 1) + 4 * (e & 1)));
    }
    reinterpret_cast<uint4*>(record)[lane] = make_uint4(v[0], v[1], v[2], v[3]);
  } else {
    // pair P = 4 t + (e >> 1) of the lane: P < 15 in dword P / 5 at bits 3 (P % 5) and 16 + 3 (P % 5);
    // pair 15 in the spare bits 15 / 31, code bit b in dword b
    uint32_t v[3] = {0, 0, 0};
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t code = q[t * 8 + e];
        const int P = 4 * t + (e >> 1), half = (e & 1) * 16;
        if (P < 15) {
          v[P / 5] |= code << (half + 3 * (P % 5));
        } else {
#pragma unroll
          for (int b = 0; b < 3; ++b) v[b] |= ((code >> b) & 1u) << (half + 15);
        }
      }
    record[lane * 3 + 0] = v[0]; record[lane * 3 + 1] = v[1]; record[lane * 3 + 2] = v[2];
  }
  const uint16_t z16 = f64_to_f16_bits(z);
  if (kq == 0) record[kCodeDwords + r] = static_cast<uint32_t>(s16) | (static_cast<uint32_t>(z16) << 16);

  if (!valid) return;
  // layout-independent copies: one code per byte in storage order, scale and zero per (row, group)
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    unsigned long long bytes = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) bytes |= static_cast<unsigned long long>(q[t * 8 + e]) << (8 * e);
    *reinterpret_cast<unsigned long long*>(codes + static_cast<size_t>(n) * C + g * kGroup + t * kKStep + kq * 8) = bytes;
  }
  if (kq == 0) {
    scales[static_cast<size_t>(n) * G + g] = s16;
    zeros[static_cast<size_t>(n) * G + g] = z16;
  }
}

// The fp16 salient block: one wave per (tile, k-step of 32 salient channels).  Lane l owns row
// 16 tile + l % 16 and the eight storage columns 32 ks + 8 (l / 16) + e.
__global__ __launch_bounds__(256) void salient_pack_kernel(const uint16_t* __restrict__ what, int N, int D,
                                                           int K, int ntiles,
                                                           const int32_t* __restrict__ perm,
                                                           uint4* __restrict__ wS, uint16_t* __restrict__ W_S,
                                                           unsigned* __restrict__ flag) {
  const int ks_s = K / kKStep;
  const int lane = threadIdx.x & 63;
  const int item = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= ntiles * ks_s) return;
  const int tile = item / ks_s, ks = item - tile * ks_s;
  const int r = lane & 15, kq = lane >> 4;
  const int n = tile * kTileN + r;
  uint16_t h[8];
  bool bad = false;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    h[e] = n < N ? what[static_cast<size_t>(n) * D + perm[ks * kKStep + kq * 8 + e]] : uint16_t{0};
    bad |= ((h[e] >> 10) & 31) == 31;
  }
  if (bad) atomicOr(flag, 1u);
  const uint4 v = make_uint4(h[0] | (uint32_t(h[1]) << 16), h[2] | (uint32_t(h[3]) << 16),
                             h[4] | (uint32_t(h[5]) << 16), h[6] | (uint32_t(h[7]) << 16));
  wS[static_cast<size_t>(item) * 64 + lane] = v;
  if (n < N) *reinterpret_cast<uint4*>(W_S + static_cast<size_t>(n) * K + ks * kKStep + kq * 8) = v;
}

// fp16(Q) in the fragment order of the run-time rotation kernels, from the fp32 rotation.
//   dense:      [D/16 tiles][D/32 k-steps][64 lanes][8]: Q[32 ks + 8 (l/16) + e][perm[16 t + l%16]]
//               (rows of the "weight" Q^T already in storage order)
//   head-wise:  [H][8 column tiles][4 k-steps][64 lanes][8]: Q_h[32 t + 8 (l/16) + e][16 ct + l%16]
__global__ __launch_bounds__(256) void rotation_image_kernel(const float* __restrict__ Q, int D, int headwise,
                                                             const int32_t* __restrict__ perm,
                                                             uint4* __restrict__ qf, size_t total) {
  const size_t idx = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= total) return;
  const int lane = static_cast<int>(idx & 63), r = lane & 15, kq = lane >> 4;
  const size_t frag = idx >> 6;
  _Float16 h[8];
  if (headwise) {
    const int t = static_cast<int>(frag & 3), ct = static_cast<int>((frag >> 2) & 7);
    const size_t head = frag >> 5;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      h[e] = static_cast<_Float16>(Q[(head * kHeadDim + t * kKStep + kq * 8 + e) * kHeadDim + ct * 16 + r]);
  } else {
    const int ks_n = D / kKStep;
    const int ks = static_cast<int>(frag % ks_n);
    const size_t tile = frag / ks_n;
    const int ch = perm[tile * kTileN + r];
#pragma unroll
    for (int e = 0; e < 8; ++e)
      h[e] = static_cast<_Float16>(Q[static_cast<size_t>(ks * kKStep + kq * 8 + e) * D + ch]);
  }
  uint32_t wv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    wv[i] = __builtin_bit_cast(uint16_t, h[2 * i]) | (uint32_t(__builtin_bit_cast(uint16_t, h[2 * i + 1])) << 16);
  qf[idx] = make_uint4(wv[0], wv[1], wv[2], wv[3]);
}

static int quant_fail(hipError_t e, const char* what) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  return ROSAQ_ERR_HIP;
}

int launch_quantize_pack(const QuantPackArgs& a, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int ntiles = ((a.N + 127) / 128) * 8;
  const int ks_s = a.K / kKStep, G = (a.D - a.K) / kGroup;
  const uint16_t* what = static_cast<const uint16_t*>(a.what16);
  unsigned* flag = static_cast<unsigned*>(a.flag);
  if (ks_s > 0) {
    const int items = ntiles * ks_s;
    hipLaunchKernelGGL(salient_pack_kernel, dim3((items + 3) / 4), dim3(256), 0, st, what, a.N, a.D, a.K, ntiles,
                       a.perm, static_cast<uint4*>(a.wS_image), static_cast<uint16_t*>(a.W_S), flag);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return quant_fail(e, "salient_pack_kernel launch");
  }
  if (G > 0) {
    const int recs = ntiles * G;
    if (a.bits == 4)
      hipLaunchKernelGGL(quantize_pack_kernel<4>, dim3((recs + 3) / 4), dim3(256), 0, st, what, a.N, a.D, a.K, G,
                         ntiles, a.perm, static_cast<uint32_t*>(a.wq_image), static_cast<uint8_t*>(a.codes),
                         static_cast<uint16_t*>(a.scales), static_cast<uint16_t*>(a.zeros), flag);
    else
      hipLaunchKernelGGL(quantize_pack_kernel<3>, dim3((recs + 3) / 4), dim3(256), 0, st, what, a.N, a.D, a.K, G,
                         ntiles, a.perm, static_cast<uint32_t*>(a.wq_image), static_cast<uint8_t*>(a.codes),
                         static_cast<uint16_t*>(a.scales), static_cast<uint16_t*>(a.zeros), flag);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return quant_fail(e, "quantize_pack_kernel launch");
  }
  return ROSAQ_OK;
}

int launch_rotation_image(const void* Q_dev, int D, int headwise, const int32_t* perm_dev, void* qf_image,
                          void* stream) {
  const size_t total = headwise ? static_cast<size_t>(D / kHeadDim) * 8 * 4 * 64
                                : static_cast<size_t>(D / kTileN) * (D / kKStep) * 64;
  hipLaunchKernelGGL(rotation_image_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const float*>(Q_dev), D, headwise, perm_dev,
                     static_cast<uint4*>(qf_image), total);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? ROSAQ_OK : quant_fail(e, "rotation_image_kernel launch");
}

}  // namespace rosaq
