// gfx950 kernels of the fused ROSAQ linear layer (Eq. 3 / Eq. 6).
//
// Data flow of one call:
//   prologue   x [M x D] fp16  ->  xhat fragments in storage order
//                NONE      gather_kernel (permutation only, R = I)
//                HEADWISE  rotate_headwise_kernel (128x128 MFMA blocks, Eq. 6)
//                FULL      gather_kernel (identity) + gemm_kernel on fp16(Q)^T
//   main       gemm_kernel: y = xhat_S W_S^T + xhat_N ((q - z) s)^T, fp32 accumulate
//
// All matrix operands are kept in "fragment order": a fragment is what one
// v_mfma_f32_16x16x32_f16 consumes, 64 lanes x 16 bytes, lane l holding 8 halves
// for (row or column l % 16, contraction indices 8*(l/16)..8*(l/16)+7).  A wave
// fetches a fragment with one global_load_dwordx4 per lane, 1 KiB contiguous.
#include <hip/hip_runtime.h>

#include "rosaq_internal.h"

namespace rosaq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ half2v as_h2(uint32_t v) { return __builtin_bit_cast(half2v, v); }
__device__ __forceinline__ half8 as_h8(uint4 v) { return __builtin_bit_cast(half8, v); }

__device__ __forceinline__ floatx4 mfma16(half8 a, half8 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Eight 4-bit codes of one dword -> eight fp16 values (q - z), exactly.
// 0x6400 | q is the fp16 number 1024 + q; 0x6400 | (q << 4) is 1024 + 16 q.
// c_lo = -(1024 + z), c_hi = -(64 + z): both subtractions are exact in fp16.
__device__ __forceinline__ half8 dequant4(uint32_t v, half2v c_lo, half2v c_hi) {
  const uint32_t kMagic = 0x64006400u;
  const half2v sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
  const uint32_t v8 = v >> 8;
  const half2v h0 = as_h2((v & 0x000f000fu) | kMagic) + c_lo;
  const half2v h1 = __builtin_elementwise_fma(as_h2((v & 0x00f000f0u) | kMagic), sixteenth, c_hi);
  const half2v h2 = as_h2((v8 & 0x000f000fu) | kMagic) + c_lo;
  const half2v h3 = __builtin_elementwise_fma(as_h2((v8 & 0x00f000f0u) | kMagic), sixteenth, c_hi);
  return half8{h0.x, h0.y, h1.x, h1.y, h2.x, h2.y, h3.x, h3.y};
}

// Eight 3-bit codes of k-step t: low two bits from the 2-bit plane dword `lo`
// (fields 4*(t&1)+i), high bit from the 1-bit plane dword `hi` (fields 4*t+i).
__device__ __forceinline__ half8 dequant3(uint32_t lo, uint32_t hi, int t, half2v c_lo) {
  const uint32_t kMagic = 0x64006400u;
  half2v h[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t a = (lo >> (2 * (4 * (t & 1) + i))) & 0x00030003u;
    const uint32_t b = ((hi >> (4 * t + i)) & 0x00010001u) << 2;
    h[i] = as_h2(kMagic | a | b) + c_lo;
  }
  return half8{h[0].x, h[0].y, h[1].x, h[1].y, h[2].x, h[2].y, h[3].x, h[3].y};
}

struct GemmDev {
  const uint4* xf;
  const uint4* wS;
  const uint32_t* wq;
  const uint32_t* sz;
  float4* partial;
  uint32_t* counters;
  _Float16* out;
  int64_t ldo;
  int M, N, ks_s, G, KS, KS_out, splits, out_frag, chunks, units;
};

// Store one accumulator fragment: lane holds rows 4*(lane/16)+i, column lane%16.
__device__ __forceinline__ void store_fragment(const GemmDev& p, float4 v, int mb, int mt, int tile,
                                               int lane) {
  const int n = tile * kTileN + (lane & 15);
  if (n >= p.N) return;
  const float vv[4] = {v.x, v.y, v.z, v.w};
  if (!p.out_frag) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = mb * kMBlock + mt * 16 + 4 * (lane >> 4) + i;
      if (m < p.M) p.out[static_cast<int64_t>(m) * p.ldo + n] = static_cast<_Float16>(vv[i]);
    }
  } else {
    const int ks = n >> 5, j = (n >> 3) & 3, e = n & 7;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int lane2 = 4 * (lane >> 4) + i + 16 * j;
      const size_t off =
          (((static_cast<size_t>(mb) * p.KS_out + ks) * 4 + mt) * 64 + lane2) * 8 + e;
      p.out[off] = static_cast<_Float16>(vv[i]);
    }
  }
}

// y tile [64 x NT*16] for a range of contraction "units": the first ks_s units are
// fp16 k-steps (32 channels each, the salient group of Eq. 3), the next G units
// are low-bit groups (128 channels each).  A workgroup owns one channel chunk and
// one split of the unit range; its waves take units round-robin, accumulate in
// fp32 registers, and are summed through LDS in a fixed order.  With splits > 1
// workgroups park their tile in `partial` and the last one to arrive adds the
// tiles in split order, so the result does not depend on scheduling.
template <int BITS, int MT, int NT, int WPB>
__global__ __launch_bounds__(WPB * 64) void gemm_kernel(GemmDev p) {
  __shared__ float4 red[WPB][NT * MT][64];
  __shared__ int s_last;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int mb = blockIdx.y;
  // Workgroups go to the 8 XCDs round-robin by linear id: keep all splits of one
  // channel chunk on one XCD so their partial tiles meet in that XCD's L2.
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int chunk = xcd + 8 * (local / p.splits);
  const int split = local % p.splits;
  if (chunk >= p.chunks) return;
  const int tile0 = chunk * NT;
  const int u0 = static_cast<int>(static_cast<int64_t>(p.units) * split / p.splits);
  const int u1 = static_cast<int>(static_cast<int64_t>(p.units) * (split + 1) / p.splits);

  floatx4 acc[NT][MT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

  const uint4* xf = p.xf + static_cast<size_t>(mb) * p.KS * 4 * 64 + lane;

  for (int u = u0 + wave; u < u1; u += WPB) {
    if (u < p.ks_s) {
      half8 a[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) a[mt] = as_h8(xf[(static_cast<size_t>(u) * 4 + mt) * 64]);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const half8 b = as_h8(p.wS[(static_cast<size_t>(tile0 + nt) * p.ks_s + u) * 64 + lane]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = mfma16(a[mt], b, acc[nt][mt]);
      }
    } else {
      const int g = u - p.ks_s;
      const int ks0 = p.ks_s + 4 * g;
      // issue the weight loads first: they are the HBM stream
      uint32_t cw[NT][4];
      uint32_t szv[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const size_t fi = (static_cast<size_t>(tile0 + nt) * p.G + g) * 64 + lane;
        if (BITS == 4) {
          const uint4 c = reinterpret_cast<const uint4*>(p.wq)[fi];
          cw[nt][0] = c.x; cw[nt][1] = c.y; cw[nt][2] = c.z; cw[nt][3] = c.w;
        } else {
          cw[nt][0] = p.wq[fi * 3 + 0];
          cw[nt][1] = p.wq[fi * 3 + 1];
          cw[nt][2] = p.wq[fi * 3 + 2];
          cw[nt][3] = 0;
        }
        szv[nt] = p.sz[(static_cast<size_t>(tile0 + nt) * p.G + g) * 16 + (lane & 15)];
      }
      half8 a[4][MT];
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          a[t][mt] = as_h8(xf[(static_cast<size_t>(ks0 + t) * 4 + mt) * 64]);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const half2v sz2 = as_h2(szv[nt]);
        const float s = static_cast<float>(sz2.x);
        const _Float16 z = sz2.y;
        const _Float16 clo = -(z + (_Float16)1024.0f);
        const _Float16 chi = -(z + (_Float16)64.0f);
        const half2v c_lo = {clo, clo}, c_hi = {chi, chi};
        floatx4 tmp[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) tmp[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          half8 b;
          if (BITS == 4) b = dequant4(cw[nt][t], c_lo, c_hi);
          else b = dequant3(cw[nt][t >> 1], cw[nt][2], t, c_lo);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) tmp[mt] = mfma16(a[t][mt], b, tmp[mt]);
        }
        // the group scale is applied once per 128 channels, in fp32
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nt][mt] += s * tmp[mt];
      }
    }
  }

  // ---- reduce the waves of this workgroup through LDS, fixed order ----------------
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const floatx4 v = acc[nt][mt];
      red[wave][nt * MT + mt][lane] = make_float4(v[0], v[1], v[2], v[3]);
    }
  __syncthreads();

  constexpr int kSlots = NT * MT;           // accumulator fragments per tile
  constexpr int kPerWave = (kSlots + WPB - 1) / WPB;
  float4 sum[kPerWave];
#pragma unroll
  for (int i = 0; i < kPerWave; ++i) {
    const int slot = wave + i * WPB;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (slot < kSlots) {
      v = red[0][slot][lane];
#pragma unroll
      for (int w = 1; w < WPB; ++w) {
        const float4 o = red[w][slot][lane];
        v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
      }
    }
    sum[i] = v;
  }

  if (p.splits == 1) {
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      const int slot = wave + i * WPB;
      if (slot < kSlots) store_fragment(p, sum[i], mb, slot % MT, tile0 + slot / MT, lane);
    }
    return;
  }

  // ---- split-K across workgroups: park, count, last arrival sums in split order ----
  const size_t tile_id = static_cast<size_t>(mb) * p.chunks + chunk;
  float4* mine = p.partial + (tile_id * p.splits + split) * (kSlots * 64);
#pragma unroll
  for (int i = 0; i < kPerWave; ++i) {
    const int slot = wave + i * WPB;
    if (slot < kSlots) mine[slot * 64 + lane] = sum[i];
  }
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t old = atomicAdd(&p.counters[tile_id], 1u);
    s_last = (old == static_cast<uint32_t>(p.splits) - 1u);
  }
  __syncthreads();
  if (!s_last) return;
  __threadfence();
  const float4* all = p.partial + tile_id * p.splits * (kSlots * 64);
#pragma unroll
  for (int i = 0; i < kPerWave; ++i) {
    const int slot = wave + i * WPB;
    if (slot >= kSlots) continue;
    float4 v = all[slot * 64 + lane];
    for (int s = 1; s < p.splits; ++s) {
      const float4 o = all[(static_cast<size_t>(s) * kSlots + slot) * 64 + lane];
      v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
    }
    store_fragment(p, v, mb, slot % MT, tile0 + slot / MT, lane);
  }
  if (threadIdx.x == 0) p.counters[tile_id] = 0u;   // ready for the next call
}

// xhat fragments from x by a column permutation (or identity): the prologue of
// the rotation-less layer and of the dense rotation.
__global__ __launch_bounds__(256) void gather_kernel(const _Float16* __restrict__ x, int64_t ldx,
                                                     int M, int KS, const int32_t* __restrict__ perm,
                                                     uint4* __restrict__ xf, int total) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int lane = idx & 63, mt = (idx >> 6) & 3;
  const int ks = (idx >> 8) % KS, mb = (idx >> 8) / KS;
  const int m = mb * kMBlock + mt * 16 + (lane & 15);
  const int p0 = ks * kKStep + (lane >> 4) * 8;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (m < M) {
    const _Float16* row = x + static_cast<int64_t>(m) * ldx;
    if (perm == nullptr) {
      v = *reinterpret_cast<const uint4*>(row + p0);
    } else {
      uint16_t h[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) h[e] = __builtin_bit_cast(uint16_t, row[perm[p0 + e]]);
      v.x = h[0] | (uint32_t(h[1]) << 16); v.y = h[2] | (uint32_t(h[3]) << 16);
      v.z = h[4] | (uint32_t(h[5]) << 16); v.w = h[6] | (uint32_t(h[7]) << 16);
    }
  }
  xf[idx] = v;
}

// Head-wise rotation (Eq. 6): per head h and 64-row block, xhat_h = x_h fp16(Q_h)
// as 4 x 8 MFMA tiles, scattered to the storage position of each rotated channel.
__global__ __launch_bounds__(256) void rotate_headwise_kernel(
    const _Float16* __restrict__ x, int64_t ldx, int M, int KS, const uint4* __restrict__ qh,
    const int32_t* __restrict__ pos, _Float16* __restrict__ xf) {
  const int lane = threadIdx.x & 63;
  const int mt = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = blockIdx.x, mb = blockIdx.y;
  const int m = mb * kMBlock + mt * 16 + (lane & 15);
  half8 a[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (m < M)
      v = *reinterpret_cast<const uint4*>(x + static_cast<int64_t>(m) * ldx + h * kHeadDim +
                                          t * kKStep + (lane >> 4) * 8);
    a[t] = as_h8(v);
  }
#pragma unroll
  for (int ct = 0; ct < 8; ++ct) {
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 4; ++t)
      acc = mfma16(a[t], as_h8(qh[((static_cast<size_t>(h) * 8 + ct) * 4 + t) * 64 + lane]), acc);
    const int p = pos[h * kHeadDim + ct * 16 + (lane & 15)];
    const int ks = p >> 5, j = (p >> 3) & 3, e = p & 7;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int lane2 = 4 * (lane >> 4) + i + 16 * j;
      xf[(((static_cast<size_t>(mb) * KS + ks) * 4 + mt) * 64 + lane2) * 8 + e] =
          static_cast<_Float16>(acc[i]);
    }
  }
}

// ---- launchers ------------------------------------------------------------------
static int hip_fail(hipError_t e, const char* what) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  return ROSAQ_ERR_HIP;
}

int pick_splits(int M, int N, int units) {
  const int ntiles = ((N + 127) / 128) * 8;
  const int chunks = ntiles / 4;
  const int mblocks = (M + kMBlock - 1) / kMBlock;
  const int wgs = chunks * mblocks;
  int s = (256 + wgs - 1) / wgs;            // aim at one workgroup per compute unit
  s = std::min(s, std::max(1, units / 4));  // keep at least one unit per wave
  return std::max(1, std::min(s, 64));
}

template <int BITS, int MT, int WPB>
static int launch_gemm_t(const GemmDev& d, int mblocks, hipStream_t st) {
  const int xblocks = ((d.chunks + 7) / 8) * 8 * d.splits;
  hipLaunchKernelGGL((gemm_kernel<BITS, MT, 4, WPB>), dim3(xblocks, mblocks), dim3(WPB * 64), 0, st, d);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? ROSAQ_OK : hip_fail(e, "gemm_kernel launch");
}

int launch_gemm(const GemmArgs& a, int wpb_override, void* stream) {
  GemmDev d;
  d.xf = static_cast<const uint4*>(a.xf);
  d.wS = static_cast<const uint4*>(a.wS);
  d.wq = static_cast<const uint32_t*>(a.wq);
  d.sz = static_cast<const uint32_t*>(a.sz);
  d.partial = reinterpret_cast<float4*>(a.partial);
  d.counters = a.counters;
  d.out = static_cast<_Float16*>(a.out);
  d.ldo = a.ldo;
  d.M = a.M; d.N = a.N; d.ks_s = a.ks_s; d.G = a.G; d.KS = a.KS; d.KS_out = a.KS_out;
  d.splits = a.splits; d.out_frag = a.out_frag;
  d.chunks = a.ntiles / 4;
  d.units = a.ks_s + a.G;
  const int mblocks = (a.M + kMBlock - 1) / kMBlock;
  const int mt = a.M <= 16 ? 1 : (a.M <= 32 ? 2 : 4);
  const int bits = a.G == 0 ? 4 : a.bits;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool w8 = wpb_override == 8;
#define ROSAQ_GEMM_CASE(B, T)                                              \
  if (bits == B && mt == T)                                               \
    return w8 ? launch_gemm_t<B, T, 8>(d, mblocks, st) : launch_gemm_t<B, T, 4>(d, mblocks, st);
  ROSAQ_GEMM_CASE(4, 1) ROSAQ_GEMM_CASE(4, 2) ROSAQ_GEMM_CASE(4, 4)
  ROSAQ_GEMM_CASE(3, 1) ROSAQ_GEMM_CASE(3, 2) ROSAQ_GEMM_CASE(3, 4)
#undef ROSAQ_GEMM_CASE
  set_error("no kernel for this bits / M combination");
  return ROSAQ_ERR_ARG;
}

int launch_gather(const void* x, int64_t ldx, int M, int D, const int32_t* perm_dev, void* xf,
                  void* stream) {
  const int KS = D / kKStep, mblocks = (M + kMBlock - 1) / kMBlock;
  const int total = mblocks * KS * 256;
  hipLaunchKernelGGL(gather_kernel, dim3((total + 255) / 256), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const _Float16*>(x), ldx, M, KS,
                     perm_dev, static_cast<uint4*>(xf), total);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? ROSAQ_OK : hip_fail(e, "gather_kernel launch");
}

int launch_rotate_headwise(const void* x, int64_t ldx, int M, int D, const void* qh,
                           const int32_t* pos_dev, void* xf, void* stream) {
  const int H = D / kHeadDim, mblocks = (M + kMBlock - 1) / kMBlock;
  hipLaunchKernelGGL(rotate_headwise_kernel, dim3(H, mblocks), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const _Float16*>(x), ldx, M,
                     D / kKStep, static_cast<const uint4*>(qh), pos_dev,
                     static_cast<_Float16*>(xf));
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? ROSAQ_OK : hip_fail(e, "rotate_headwise_kernel launch");
}

}  // namespace rosaq
