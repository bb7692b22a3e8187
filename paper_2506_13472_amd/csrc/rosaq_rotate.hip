// Dense rotation xhat = x fp16(Q) for calls of up to 64 rows (Eq. 1 with the layer-wise PCA
// rotation of Sec. 3.1): a skinny fp16 contraction whose cost is the stream of fp16(Q) from HBM
// (2 D^2 bytes: 33.5 MB at D = 4096, 52 MB at D = 5120).
//
// An alternative to the single output-stationary launch, selected with rosaq_tune("rot_splits", n).
// Two launches, no workgroup waits for another and nothing is exchanged inside a launch:
//   rotate_slab_kernel  one workgroup owns a slab of the contraction (a run of k-steps) and a
//                       chunk of eight 16-channel tiles.  Its slab of x (all rows) is read once,
//                       row-major and in place, and kept in LDS; every wave owns one tile and
//                       requests all its Q fragments of the slab (contiguous along k) before it
//                       uses any.  A compute unit so pulls 64 rows x slab of x instead of
//                       64 rows x D, which is what bounded the output-stationary launch.  The
//                       partial tiles leave as plain fp32 stores.
//   rotate_sum_kernel   adds the slabs of a tile in slab order (deterministic) and writes xhat as
//                       fp16 MFMA A fragments in 16-byte pieces.
// The end of the first launch publishes the partial tiles to the second: no fences, no tickets.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <string>

#include "rosaq_internal.h"

namespace rosaq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

struct RotSlabDev {
  const _Float16* x;     // [M x D] row-major
  int64_t ldx;
  int M;
  const uint4* qf;       // fp16(Q)^T fragments [tiles][KS][64 lanes], rows in storage order
  int KS, tiles, splits;
  float4* part;          // [splits][tiles][4 row tiles][64 lanes]
  unsigned* zero_ptr;    // words cleared for the launches that follow (may be null)
  int zero_count;
};

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global
// load in flight (its fences cover all address spaces), which here would wait for the whole
// Q slab before the first multiply.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// KSL: most k-steps a slab may hold (LDS: KSL x 4 KiB).  Eight waves, one 16-channel tile each.
// (Two waves per tile, each with half of a slab twice as long -- half the partial tiles -- was
// measured at D = 4096: 13.0 us against 11.3 for this launch; the slab of x a compute unit pulls
// and holds doubles.)
template <int KSL>
__global__ __launch_bounds__(512) void rotate_slab_kernel(RotSlabDev p) {
  __shared__ uint4 a_lds[KSL][4][64];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int S = p.splits;
  // consecutive workgroups go to consecutive XCDs: with the slab as the fast index, a slab of x
  // is asked for by as few L2s as possible (one each when S = 8)
  const int split = blockIdx.x % S, chunk = blockIdx.x / S;
  if (p.zero_ptr != nullptr)
    for (int i = blockIdx.x * 512 + tid; i < p.zero_count; i += gridDim.x * 512) p.zero_ptr[i] = 0u;
  const int k_lo = static_cast<int>(static_cast<long long>(split) * p.KS / S);
  const int k_hi = static_cast<int>(static_cast<long long>(split + 1) * p.KS / S);
  const int nk = k_hi - k_lo;                      // 1 .. KSL (the host checks)

  // Nothing below that loads is conditional: a branch around a load makes the number of loads
  // in flight depend on the path taken, and the wait before the next use then drains them all.
  // A k-step past the end of the slab re-reads the last one and is never multiplied; a row past
  // M re-reads row M - 1 (its rows of xhat are never used by the GEMM that follows).
  constexpr int kPerThread = KSL / 2;              // KSL x 256 sixteen-byte pieces over 512 threads
  uint4 xr[kPerThread];
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const int idx = tid + 512 * i;
    const int kk = idx >> 8, mt = (idx >> 6) & 3, l = idx & 63;
    const int m = mt * 16 + (l & 15);
    const int mc = m < p.M ? m : p.M - 1, kc = kk < nk ? kk : nk - 1;
    xr[i] = *reinterpret_cast<const uint4*>(p.x + static_cast<int64_t>(mc) * p.ldx +
                                            static_cast<int64_t>(k_lo + kc) * kKStep + (l >> 4) * 8);
  }
  const int T = chunk * 8 + wave;
  const uint4* bptr = p.qf + (static_cast<size_t>(T) * p.KS + k_lo) * 64 + lane;
  // Register slot kk holds k-step (kk + skew) % nk of the slab.  The Q fragments of the waves of
  // a launch lie a power-of-two number of KiB apart when D is a power of two: walking them all
  // from the same k would keep the whole chip on a few memory channels at a time.
  const int skew = static_cast<int>((blockIdx.x * 8u + wave) * 5u % static_cast<unsigned>(nk));
  auto step_of = [&](int kk) { const int v = kk + skew; return kk < nk ? (v >= nk ? v - nk : v) : skew; };
  uint4 b[KSL];
#pragma unroll
  for (int kk = 0; kk < KSL; ++kk) b[kk] = bptr[static_cast<size_t>(step_of(kk)) * 64];
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const int idx = tid + 512 * i;
    a_lds[idx >> 8][(idx >> 6) & 3][idx & 63] = xr[i];
  }
  lds_barrier();

  floatx4 acc[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < KSL; ++kk) {
    if (kk < nk) {                                 // uniform; no loads inside
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a_lds[step_of(kk)][mt][lane]),
                                                          __builtin_bit_cast(half8, b[kk]), acc[mt], 0, 0, 0);
    }
  }
  float4* out = p.part + ((static_cast<size_t>(split) * p.tiles + T) * 4) * 64 + lane;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
    out[mt * 64] = make_float4(acc[mt][0], acc[mt][1], acc[mt][2], acc[mt][3]);
}

// One workgroup per 16-channel tile, one wave per 16-row tile.  A lane of the accumulator layout
// holds rows 4 (lane / 16) + i of channel lane % 16; the A fragment the GEMM reads wants, per
// lane, eight consecutive channels of one row: the tile turns through LDS and leaves as 32
// sixteen-byte stores per wave.
__global__ __launch_bounds__(256) void rotate_sum_kernel(const float4* __restrict__ part, int splits,
                                                         int tiles, _Float16* __restrict__ xf) {
  __shared__ _Float16 t_lds[4][16][16 + 8];        // [row tile][row][channel], rows padded
  const int tid = threadIdx.x, lane = tid & 63, mt = tid >> 6;
  const int T = blockIdx.x;
  const float4* src = part + (static_cast<size_t>(T) * 4 + mt) * 64 + lane;
  const size_t pitch = static_cast<size_t>(tiles) * 4 * 64;
  // eight loads in flight, none under a condition (a slab past the end re-reads the last one and
  // is dropped when the values are added)
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s0 = 0; s0 < splits; s0 += 8) {
    float4 o[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) o[q] = src[static_cast<size_t>(s0 + q < splits ? s0 + q : splits - 1) * pitch];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const bool use = s0 + q < splits;
      v.x += use ? o[q].x : 0.f; v.y += use ? o[q].y : 0.f;
      v.z += use ? o[q].z : 0.f; v.w += use ? o[q].w : 0.f;
    }
  }
  const int r0 = 4 * (lane >> 4), c = lane & 15;
  t_lds[mt][r0 + 0][c] = static_cast<_Float16>(v.x);
  t_lds[mt][r0 + 1][c] = static_cast<_Float16>(v.y);
  t_lds[mt][r0 + 2][c] = static_cast<_Float16>(v.z);
  t_lds[mt][r0 + 3][c] = static_cast<_Float16>(v.w);
  __syncthreads();
  if (lane < 32) {
    // storage channels 16 T + 8 jj .. + 7 of row `row`: k-step T / 2, k-slice j = 2 (T % 2) + jj
    const int jj = lane >> 4, row = lane & 15;
    const uint4 h = *reinterpret_cast<const uint4*>(&t_lds[mt][row][8 * jj]);
    const int ks = T >> 1, j = 2 * (T & 1) + jj;
    *reinterpret_cast<uint4*>(xf + ((static_cast<size_t>(ks) * 4 + mt) * 64 + 16 * j + row) * 8) = h;
  }
}

static int rot_fail(hipError_t e, const char* what) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  return ROSAQ_ERR_HIP;
}

// Checks a slab count for a D x D rotation: every slab must fit the LDS (32 k-steps).  Returns the
// count, or 0 when it does not fit (the caller then keeps the single launch).
int pick_rotate_slabs(int D, int forced) {
  const int KS = D / kKStep;
  if (forced < 1 || forced > kMaxSplits || forced > KS) return 0;
  return (KS + forced - 1) / forced <= 32 ? forced : 0;
}

size_t rotate_slab_part_bytes(int D, int slabs) {
  return static_cast<size_t>(slabs) * (D / kTileN) * 4 * 64 * sizeof(float4);
}

int launch_rotate_slabs(const void* x, int64_t ldx, int M, int D, const void* qf, int slabs, void* part,
                        void* xf_out, void* zero_ptr, int zero_count, void* stream) {
  RotSlabDev d;
  d.x = static_cast<const _Float16*>(x); d.ldx = ldx; d.M = M;
  d.qf = static_cast<const uint4*>(qf);
  d.KS = D / kKStep; d.tiles = D / kTileN; d.splits = slabs;
  d.part = static_cast<float4*>(part);
  d.zero_ptr = static_cast<unsigned*>(zero_ptr); d.zero_count = zero_count;
  const int ksl = slabs > 0 ? (d.KS + slabs - 1) / slabs : 0;
  if (M < 1 || M > kMBlock || slabs < 1 || slabs > d.KS || ksl > 32 || D % 128 != 0) {
    set_error("launch_rotate_slabs: shape outside what the kernel was built for");
    return ROSAQ_ERR_SHAPE;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 grid((D / 128) * slabs);
  if (ksl <= 16) hipLaunchKernelGGL(rotate_slab_kernel<16>, grid, dim3(512), 0, st, d);
  else hipLaunchKernelGGL(rotate_slab_kernel<32>, grid, dim3(512), 0, st, d);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return rot_fail(e, "rotate_slab_kernel launch");
  hipLaunchKernelGGL(rotate_sum_kernel, dim3(d.tiles), dim3(256), 0, st, static_cast<const float4*>(part),
                     slabs, d.tiles, static_cast<_Float16*>(xf_out));
  e = hipGetLastError();
  return e == hipSuccess ? ROSAQ_OK : rot_fail(e, "rotate_sum_kernel launch");
}

}  // namespace rosaq
