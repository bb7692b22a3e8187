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

#include <algorithm>
#include <cmath>

#include "rosaq_device.h"
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

// (v & mask) | magic in one VALU op.  The compiler splits this into v_and + v_or with
// two literals; VOP3 on gfx9 takes no literal, so the mask goes in an SGPR and the
// magic constant in a VGPR.
__device__ __forceinline__ uint32_t and_or(uint32_t v, uint32_t mask, uint32_t magic) {
  uint32_t r;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "s"(mask), "v"(magic));
  return r;
}

// Eight 4-bit codes of one dword -> eight fp16 values (q - z), exactly.
// 0x6400 | q is the fp16 number 1024 + q; 0x6400 | (q << 4) is 1024 + 16 q.
// c_lo = -(1024 + z), c_hi = -(64 + z): both subtractions are exact in fp16.
__device__ __forceinline__ half8 dequant4(uint32_t v, half2v c_lo, half2v c_hi) {
  const uint32_t kMagic = 0x64006400u;
  const half2v sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
  const uint32_t v8 = v >> 8;
  const half2v h0 = as_h2(and_or(v, 0x000f000fu, kMagic)) + c_lo;
  const half2v h1 = __builtin_elementwise_fma(as_h2(and_or(v, 0x00f000f0u, kMagic)), sixteenth, c_hi);
  const half2v h2 = as_h2(and_or(v8, 0x000f000fu, kMagic)) + c_lo;
  const half2v h3 = __builtin_elementwise_fma(as_h2(and_or(v8, 0x00f000f0u, kMagic)), sixteenth, c_hi);
  return half8{h0.x, h0.y, h1.x, h1.y, h2.x, h2.y, h3.x, h3.y};
}

// Eight 3-bit codes of k-step t -> eight fp16 values (q - z), exactly.  The 16 fp16 pairs
// P = 4 t + i of a lane's group sit in three dwords: pair P < 15 in dword P / 5 at bit
// offset 3 (P % 5) of both halves, pair 15 in the spare bits 15 / 31 (code bit b in dword b).
// A field at offset o <= 6 is masked straight into the mantissa: 0x6400 | (q << o) is the
// fp16 number 1024 + 2^o q, and one fma with 2^-o and -(1024 * 2^-o + z) gives q - z; the
// fields at offsets 9 and 12 take one shared shift first.  10 instructions per k-step.
struct Dq3 { half2v c0, c3, c6; };   // -(1024 + z), -(128 + z), -(16 + z)
__device__ __forceinline__ Dq3 dq3_consts(_Float16 z) {
  const _Float16 a = -(z + (_Float16)1024.0f), b = -(z + (_Float16)128.0f), c = -(z + (_Float16)16.0f);
  return Dq3{half2v{a, a}, half2v{b, b}, half2v{c, c}};
}
__device__ __forceinline__ half8 dequant3(uint32_t w0, uint32_t w1, uint32_t w2, int t, const Dq3& k) {
  const uint32_t kMagic = 0x64006400u;
  const half2v eighth = {(_Float16)0.125f, (_Float16)0.125f};
  const half2v sixty4th = {(_Float16)0.015625f, (_Float16)0.015625f};
  const uint32_t w[3] = {w0, w1, w2};
  half2v h[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int P = 4 * t + i;
    if (P < 15) {
      const int s = P % 5;
      const uint32_t src = s < 3 ? w[P / 5] : w[P / 5] >> 9;
      const int o = s < 3 ? s : s - 3;
      if (o == 0) h[i] = as_h2(and_or(src, 0x00070007u, kMagic)) + k.c0;
      else if (o == 1) h[i] = __builtin_elementwise_fma(as_h2(and_or(src, 0x00380038u, kMagic)), eighth, k.c3);
      else h[i] = __builtin_elementwise_fma(as_h2(and_or(src, 0x01c001c0u, kMagic)), sixty4th, k.c6);
    } else {
      uint32_t r = and_or(w0 >> 15, 0x00010001u, kMagic);
      r = and_or(w1 >> 14, 0x00020002u, r);
      r = and_or(w2 >> 13, 0x00040004u, r);
      h[i] = as_h2(r) + k.c0;
    }
  }
  return half8{h[0].x, h[0].y, h[1].x, h[1].y, h[2].x, h[2].y, h[3].x, h[3].y};
}

// 12-byte lane record of the INT3 image, read with one global_load_dwordx3
struct __attribute__((aligned(4))) Code3 { uint32_t w0, w1, w2; };

// One packed layer inside a launch.  A launch covers up to kMaxBatch layers that
// share the rotated input (e.g. the q, k, v projections of one attention block).
struct GemmSeg {
  const uint4* wS;
  const uint32_t* wq;   // records: code fragment (256 / 192 dwords) + 16 scale|zero words
  _Float16* out;
  int64_t ldo;
  int N;
  int tile_end;      // exclusive prefix sum of the layers' valid channel tiles, ceil(N / 16)
};
struct GemmDev {
  const uint4* xf;
  const _Float16* xrow;   // all-fp16 launches only: read A fragments from row-major x instead of xf
  int64_t ldx;
  GemmSeg seg[kMaxBatch];
  int nseg;
  int M, ks_s, G, KS, KS_out, out_frag, chunks, mgroups;
  // split-K across workgroups: `splits` workgroups share one output tile, each over its own run
  // of the contraction; their fp32 partial tiles meet in `part`, and the workgroup that draws
  // the last ticket of a tile adds them up in split order and stores the result
  int splits;
  float4* part;            // [tiles][splits][MT * NT][64] float4
  unsigned* tickets;       // [tiles], zero before the launch and zero again after it
  unsigned* zero_ptr;      // words this launch clears for a later launch (may be null)
  int zero_count;
  // gated pair (two layers of equal width, unsplit): the tile list alternates layer 0 / layer 1
  // tiles of the same channels, and the epilogue stores silu(layer 0) * layer 1 to seg[0].out
  int swiglu;
  // gated pair feeding a layer without run-time rotation (out_frag == 2): the product goes
  // straight into that layer's input fragments, channel n at its storage position out_pos[n]
  const int* out_pos;
};

// Partial tiles and tickets travel between workgroups that may sit on different XCDs, whose L2
// caches do not see each other's lines.  They are therefore written and read with device-scope
// relaxed atomics (64 bits at a time), which go past the non-coherent cache levels, instead of
// a release / acquire pair, which on this chip writes back and invalidates a whole L2.
__device__ __forceinline__ void store_device_scope(float4* p, float4 v) {
  unsigned long long* q = reinterpret_cast<unsigned long long*>(p);
  const unsigned long long lo = static_cast<unsigned long long>(__builtin_bit_cast(uint32_t, v.x)) |
                                (static_cast<unsigned long long>(__builtin_bit_cast(uint32_t, v.y)) << 32);
  const unsigned long long hi = static_cast<unsigned long long>(__builtin_bit_cast(uint32_t, v.z)) |
                                (static_cast<unsigned long long>(__builtin_bit_cast(uint32_t, v.w)) << 32);
  __hip_atomic_store(q, lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(q + 1, hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float4 load_device_scope(const float4* p) {
  const unsigned long long* q = reinterpret_cast<const unsigned long long*>(p);
  const unsigned long long lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const unsigned long long hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float4(__builtin_bit_cast(float, static_cast<uint32_t>(lo)),
                     __builtin_bit_cast(float, static_cast<uint32_t>(lo >> 32)),
                     __builtin_bit_cast(float, static_cast<uint32_t>(hi)),
                     __builtin_bit_cast(float, static_cast<uint32_t>(hi >> 32)));
}

// Split `s` of `splits` owns the units [u_lo, u_hi) of the fp16 k-steps and [g_lo, g_hi) of the
// low-bit groups: the contraction is cut at multiples of total / splits k-steps (a group counts
// as four), each cut moved to the nearest group boundary once it lies past the fp16 k-steps.
__host__ __device__ __forceinline__ void split_cut(int s, int splits, int ks_s, int G, int& u, int& g) {
  const int total = ks_s + 4 * G;
  const int b = static_cast<int>(static_cast<long long>(s) * total / splits);
  if (b <= ks_s) { u = b; g = 0; return; }
  u = ks_s;
  g = (b - ks_s + 2) >> 2;
  if (g > G) g = G;
}

// Block -> (channel chunk, row group).  blockIdx % 8 is the XCD a workgroup lands on; each
// XCD owns the chunks congruent to its number.  Inside an XCD consecutive workgroups, which
// run at the same time, form blocks of 8 chunks x up to 4 row groups: they share the weights
// of 8 chunks and the activations of 4 row groups through that XCD's L2, instead of one
// chunk and every row group (which at large M streams the whole activation matrix through
// every L2 once per chunk).  For up to 4 row groups this is the plain order: chunk-major.
constexpr int kMapCols = 8, kMapRows = 4;
__host__ __device__ __forceinline__ bool map_block(int b, int chunks, int mgroups, int& chunk, int& mg) {
  const int xcd = b & 7, local = b >> 3;
  if (mgroups <= kMapRows) {                              // plain chunk-major order
    mg = local % mgroups;
    chunk = xcd + 8 * (local / mgroups);
    return chunk < chunks;
  }
  const int tr = kMapRows;
  const int cx = (chunks + 7) >> 3;                       // chunk slots of one XCD
  const int cols = cx < kMapCols ? cx : kMapCols;         // narrow launches: narrower blocks, less padding
  const int nbc = (cx + cols - 1) / cols;
  const int block = local / (cols * tr), inner = local - block * (cols * tr);
  const int ci = (block % nbc) * cols + inner / tr;
  mg = (block / nbc) * tr + inner % tr;
  chunk = xcd + 8 * ci;
  return ci < cx && chunk < chunks && mg < mgroups;
}
static int map_grid(int chunks, int mgroups) {
  if (mgroups <= kMapRows) return ((chunks + 7) / 8) * 8 * mgroups;
  const int tr = kMapRows;
  const int cx = (chunks + 7) / 8;
  const int cols = cx < kMapCols ? cx : kMapCols;
  const int nbc = (cx + cols - 1) / cols;
  return 8 * nbc * ((mgroups + tr - 1) / tr) * cols * tr;
}
int block_map_host(int b, int chunks, int mgroups, int* chunk, int* mg) {
  if (b < 0) return map_grid(chunks, mgroups);          // the grid size
  return map_block(b, chunks, mgroups, *chunk, *mg) ? 1 : 0;
}

// The layers of a launch are one list of channel tiles (layer 0's valid tiles, then layer 1's,
// ...): a chunk of NT consecutive tiles may end in one layer and go on in the next, so a
// batch whose layers are not a multiple of NT tiles wide still fills whole chunks.  Tile T of
// the list lies in layer `si` at local index `local`; beyond the list it maps to the tile
// after the last layer's last one, which loads clamp and stores skip.
__device__ __forceinline__ void locate_tile(const GemmDev& p, int T, int& si, int& local) {
  si = 0;
  local = T;
  if (p.nseg == 1) return;   // the common case stays cheap (uniform branch)
  if (p.swiglu) { si = T & 1; local = T >> 1; return; }
#pragma unroll
  for (int i = 1; i < kMaxBatch; ++i)
    if (i < p.nseg && T >= p.seg[i - 1].tile_end) si = i;
  local = T - (si > 0 ? p.seg[si - 1].tile_end : 0);
}

// Layer `si` of the launch, picked by compares (indexing the by-value argument with a run-time
// index would move it to scratch memory).
__device__ __forceinline__ GemmSeg pick_seg(const GemmDev& p, int si) {
  GemmSeg sg = p.seg[0];
  if (p.nseg == 1) return sg;
#pragma unroll
  for (int i = 1; i < kMaxBatch; ++i)
    if (si == i) sg = p.seg[i];
  return sg;
}

// Store one accumulator fragment of row tile `mtile` (16 rows) and channel tile T of the
// launch's tile list: lane holds rows 4*(lane/16)+i, column lane%16.
__device__ __forceinline__ void store_fragment(const GemmDev& p, float4 v, int mtile, int T, int lane) {
  int si, tile;
  locate_tile(p, T, si, tile);
  const GemmSeg sg = pick_seg(p, si);
  const int n = tile * kTileN + (lane & 15);
  if (n >= sg.N) return;
  const float vv[4] = {v.x, v.y, v.z, v.w};
  _Float16* out = sg.out;
  if (!p.out_frag) {
    const int64_t ldo = sg.ldo;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = mtile * 16 + 4 * (lane >> 4) + i;
      if (m < p.M) out[static_cast<int64_t>(m) * ldo + n] = static_cast<_Float16>(vv[i]);
    }
  } else {
    const int ks = n >> 5, j = (n >> 3) & 3, e = n & 7;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int lane2 = 4 * (lane >> 4) + i + 16 * j;
      const size_t off =
          (((static_cast<size_t>(mtile >> 2) * p.KS_out + ks) * 4 + (mtile & 3)) * 64 + lane2) * 8 + e;
      out[off] = static_cast<_Float16>(vv[i]);
    }
  }
}

// One workgroup computes a [MT*16 rows] x [NT*16 channels] tile of the output over
// the whole contraction.  The contraction is cut into "units": first ks_s fp16
// k-steps of 32 channels (the salient group of Eq. 3), then G low-bit groups of 128
// channels.  The WPB waves take units round-robin (split-K inside the workgroup),
// each streaming its weight fragments from HBM straight into registers, and are
// summed through LDS in wave order, so the result does not depend on scheduling.
// Workgroups that share a channel chunk (different row tiles) are placed on one XCD
// so that the weights are fetched from HBM once and found in that XCD's L2 after.
template <int BITS, int MT, int NT, int WPB, int DEPTH>
__global__ __launch_bounds__(WPB * 64, (DEPTH == 1 && MT * NT <= 4 ? (MT == 4 ? 2 : 4) : 1))
void gemm_kernel(GemmDev p) {
  // the waves' partial tiles meet in LDS, in one pass or (large tiles) in two halves
  constexpr int kRedPasses = WPB * NT * MT > 128 ? 2 : 1;
  constexpr int kRedNT = NT / kRedPasses;
  static_assert(NT % kRedPasses == 0, "tile split");
  __shared__ float4 red[WPB][kRedNT * MT][64];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int chunk, mg;
  // the workgroups of one output tile are neighbours on one XCD (blockIdx % 8 is the XCD)
  const int splits = p.splits;
  const int local = blockIdx.x >> 3;
  const int split = splits > 1 ? local % splits : 0;
  const int base_block = splits > 1 ? ((local / splits) << 3) | (blockIdx.x & 7) : blockIdx.x;
  if (p.zero_ptr != nullptr && blockIdx.x == 0)
    for (int i = threadIdx.x; i < p.zero_count; i += WPB * 64) p.zero_ptr[i] = 0u;
  if (!map_block(base_block, p.chunks, p.mgroups, chunk, mg)) return;
  const int tile0 = chunk * NT;   // first tile of the chunk in the launch's tile list
  const int mtile0 = mg * MT;
  // where each of the chunk's tiles lives (uniform over the workgroup): fp16 fragments and
  // low-bit records of tile nt start at wS_t[nt] and wq_t[nt]
  const uint4* wS_t[NT];
  const uint32_t* wq_t[NT];
  constexpr int kRecDwordsT = (BITS == 4 ? 256 : 192) + 16;
  if (p.nseg == 1) {   // one layer: no search, the tiles are consecutive
    const int valid = (p.seg[0].N + kTileN - 1) / kTileN;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int tile = tile0 + nt < valid ? tile0 + nt : valid - 1;   // past the end: re-read the last tile
      wS_t[nt] = p.seg[0].wS + static_cast<size_t>(tile) * p.ks_s * 64;
      wq_t[nt] = p.seg[0].wq + static_cast<size_t>(tile) * p.G * kRecDwordsT;
    }
  } else {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      int si, tile;
      locate_tile(p, tile0 + nt, si, tile);
      const GemmSeg sg = pick_seg(p, si);
      const int valid = (sg.N + kTileN - 1) / kTileN;
      if (tile >= valid) tile = valid - 1;
      wS_t[nt] = sg.wS + static_cast<size_t>(tile) * p.ks_s * 64;
      wq_t[nt] = sg.wq + static_cast<size_t>(tile) * p.G * kRecDwordsT;
    }
  }

  floatx4 acc[NT][MT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

  // xhat fragment of row tile mtile0+mt and k-step ks: xa[mt][ks * 256]
  const uint4* xa[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int mtile = mtile0 + mt;
    xa[mt] = p.xf + (static_cast<size_t>(mtile >> 2) * p.KS * 4 + (mtile & 3)) * 64 + lane;
  }
  // Skinny inputs (single row tile per workgroup): lanes whose row is beyond M skip the
  // load, so a decode step with a few rows does not pull 16 rows of padding per k-step.
  const bool row_ok = MT > 1 || mtile0 * 16 + (lane & 15) < p.M;

  // Per-wave work list: fp16 k-steps u = wave, wave + WPB, ... and low-bit groups
  // g = g_first, g_first + WPB, ... (unit ks_s + g belongs to wave (ks_s + g) % WPB).
  // DEPTH units are requested ahead of the one being multiplied, and everything a wave needs
  // first is requested before it waits for anything.  How much of that overlaps inside a wave
  // is up to the compiler's wait placement (with the refills under conditions, as here, the first
  // use of a unit waits for every load in flight); a variant with exact progressive waits was
  // measured and was not faster: the launch is bound by what the L1 / L2 path delivers per
  // compute unit, and latency is covered by the other waves.
  struct StepRegs {
    uint4 a[MT];
    uint4 b[NT];
  };
  struct GroupRegs {
    uint32_t cw[NT][4];
    uint32_t sz[NT];
    uint4 a[4][MT];
  };
  auto load_step = [&](int u, StepRegs& r) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      r.b[nt] = wS_t[nt][static_cast<size_t>(u) * 64 + lane];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      r.a[mt] = row_ok ? xa[mt][static_cast<size_t>(u) * 256] : make_uint4(0, 0, 0, 0);
  };
  auto compute_step = [&](const StepRegs& r) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        acc[nt][mt] = mfma16(as_h8(r.a[mt]), as_h8(r.b[nt]), acc[nt][mt]);
  };
  // Every workgroup walks the groups in the same order: the fp32 sum of an output element
  // is then the same whatever the tile shape or batching of the launch (starting each
  // workgroup at its own group was measured: 1-3 % faster, not worth that property).
  auto load_group = [&](int g, GroupRegs& r) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      constexpr int kCodeDwords = BITS == 4 ? 256 : 192, kRecDwords = kCodeDwords + 16;
      const uint32_t* rec = wq_t[nt] + static_cast<size_t>(g) * kRecDwords;
      if (BITS == 4) {
        const uint4 c = reinterpret_cast<const uint4*>(rec)[lane];
        r.cw[nt][0] = c.x; r.cw[nt][1] = c.y; r.cw[nt][2] = c.z; r.cw[nt][3] = c.w;
      } else {
        const Code3 c = reinterpret_cast<const Code3*>(rec)[lane];
        r.cw[nt][0] = c.w0; r.cw[nt][1] = c.w1; r.cw[nt][2] = c.w2;
        r.cw[nt][3] = 0;
      }
      r.sz[nt] = rec[kCodeDwords + (lane & 15)];
    }
    const size_t ks0 = static_cast<size_t>(p.ks_s + 4 * g);
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        r.a[t][mt] = make_uint4(0, 0, 0, 0);
        if (row_ok) r.a[t][mt] = xa[mt][(ks0 + t) * 256];
      }
  };
  auto compute_group = [&](const GroupRegs& r) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const half2v sz2 = as_h2(r.sz[nt]);
      const float s = static_cast<float>(sz2.x);
      const _Float16 z = sz2.y;
      const _Float16 clo = -(z + (_Float16)1024.0f);
      const _Float16 chi = -(z + (_Float16)64.0f);
      const half2v c_lo = {clo, clo}, c_hi = {chi, chi};
      const Dq3 k3 = dq3_consts(z);
      floatx4 tmp[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) tmp[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        half8 b;
        if (BITS == 4) b = dequant4(r.cw[nt][t], c_lo, c_hi);
        else b = dequant3(r.cw[nt][0], r.cw[nt][1], r.cw[nt][2], t, k3);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) tmp[mt] = mfma16(as_h8(r.a[t][mt]), b, tmp[mt]);
      }
      // the group scale is applied once per 128 channels, in fp32
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[nt][mt] += s * tmp[mt];
    }
  };

  const int ks_s = p.ks_s, G = p.G;
  // this workgroup's run of the contraction (everything when the launch is not split)
  int u_lo = 0, u_hi = ks_s, g_lo = 0, g_hi = G;
  if (splits > 1 && BITS != 16) {
    split_cut(split, splits, ks_s, G, u_lo, g_lo);
    split_cut(split + 1, splits, ks_s, G, u_hi, g_hi);
  }
  if constexpr (BITS == 16) {
    // All-fp16 layer (the dense rotation, or K = D): no low-bit state, so the registers
    // go to deep prefetch.  Units are runs of four k-steps; leftover k-steps go one by one.
    struct QuadRegs {
      uint4 a[4][MT];
      uint4 b[4][NT];
    };
    auto load_quad = [&](int qd, QuadRegs& r) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          r.b[t][nt] = wS_t[nt][static_cast<size_t>(4 * qd + t) * 64 + lane];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          if (p.xrow != nullptr) {
            // lane (row r, k-slice j) reads its 8 halves straight from x[m][32 (4 qd + t) + 8 j]
            const int m = (mtile0 + mt) * 16 + (lane & 15);
            r.a[t][mt] = make_uint4(0, 0, 0, 0);
            if (m < p.M)
              r.a[t][mt] = *reinterpret_cast<const uint4*>(p.xrow + static_cast<int64_t>(m) * p.ldx +
                                                           (4 * qd + t) * kKStep + (lane >> 4) * 8);
          } else {
            r.a[t][mt] = row_ok ? xa[mt][static_cast<size_t>(4 * qd + t) * 256] : make_uint4(0, 0, 0, 0);
          }
        }
      }
    };
    auto compute_quad = [&](const QuadRegs& r) {
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            acc[nt][mt] = mfma16(as_h8(r.a[t][mt]), as_h8(r.b[t][nt]), acc[nt][mt]);
    };
    // split launches cut the run of quads evenly; leftover k-steps go to the last split
    const int quads_all = ks_s >> 2;
    const int q_lo = splits > 1 ? static_cast<int>(static_cast<long long>(split) * quads_all / splits) : 0;
    const int q_hi = splits > 1 ? static_cast<int>(static_cast<long long>(split + 1) * quads_all / splits) : quads_all;
    const int nquad = q_hi - q_lo;
    // fp16 tiles are a power-of-two number of KiB apart when D is: workgroups that all walk
    // their tiles from k = 0 would camp on the same HBM channels.  Each workgroup starts
    // its walk at its own offset (the sum over k does not care where it starts).
    const int skew = nquad ? (blockIdx.x * 5) % nquad : 0;
    auto at = [&](int i) { const int v = i + skew; return q_lo + (v >= nquad ? v - nquad : v); };
    QuadRegs q[DEPTH];
    int u = wave;
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
      if (u + d * WPB < nquad) load_quad(at(u + d * WPB), q[d]);
    for (; u < nquad; u += DEPTH * WPB) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        if (u + d * WPB < nquad) {
          compute_quad(q[d]);
          if (u + (d + DEPTH) * WPB < nquad) load_quad(at(u + (d + DEPTH) * WPB), q[d]);
        }
      }
    }
    if (split == splits - 1 || splits <= 1)
      for (int st = 4 * quads_all + wave; st < ks_s; st += WPB) {
        StepRegs s0;
        load_step(st, s0);
        compute_step(s0);
      }
  } else {
  int u = u_lo + wave;
  int g = g_lo + (wave + WPB - (u_hi - u_lo) % WPB) % WPB;
  StepRegs s0, s1;
  GroupRegs r[DEPTH];
  if (u < u_hi) load_step(u, s0);
  if (u + WPB < u_hi) load_step(u + WPB, s1);
#pragma unroll
  for (int d = 0; d < DEPTH; ++d)
    if (g + d * WPB < g_hi) load_group(g + d * WPB, r[d]);
  for (; u < u_hi; u += 2 * WPB) {
    compute_step(s0);
    if (u + 2 * WPB < u_hi) load_step(u + 2 * WPB, s0);
    if (u + WPB < u_hi) {
      compute_step(s1);
      if (u + 3 * WPB < u_hi) load_step(u + 3 * WPB, s1);
    }
  }
  for (; g < g_hi; g += DEPTH * WPB) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      if (g + d * WPB < g_hi) {
        compute_group(r[d]);
        if (g + (d + DEPTH) * WPB < g_hi) load_group(g + (d + DEPTH) * WPB, r[d]);
      }
    }
  }
  }   // BITS != 16

  // ---- gated pair: out = silu(gate) * up, both sums still in fp32, one rounding to fp16 ------
  if constexpr (kRedNT % 2 == 0) {
    if (p.swiglu) {
      constexpr int kPairs = (kRedNT / 2) * MT;
      constexpr int kPairIters = (kPairs + WPB - 1) / WPB;
      const GemmSeg sg = p.seg[0];
      // storage positions of this wave's output channels in the following layer, requested before
      // the reduction so that the stores behind it do not wait for them
      int next_pos[kRedPasses][kPairIters];
      if (p.out_frag == 2) {
#pragma unroll
        for (int pass = 0; pass < kRedPasses; ++pass)
#pragma unroll
          for (int it = 0; it < kPairIters; ++it) {
            const int ps = wave + it * WPB, j = (ps < kPairs ? ps : 0) / MT;
            const int n = ((tile0 + pass * kRedNT + 2 * j) >> 1) * kTileN + (lane & 15);
            next_pos[pass][it] = p.out_pos[n < sg.N ? n : 0];
          }
      }
#pragma unroll
      for (int pass = 0; pass < kRedPasses; ++pass) {
        if (pass > 0) __syncthreads();
#pragma unroll
        for (int nt = 0; nt < kRedNT; ++nt)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const floatx4 v = acc[pass * kRedNT + nt][mt];
            red[wave][nt * MT + mt][lane] = make_float4(v[0], v[1], v[2], v[3]);
          }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < kPairIters; ++it) {
          const int ps = wave + it * WPB;
          if (ps >= kPairs) break;
          const int j = ps / MT, mt = ps - j * MT;
          float4 g = red[0][(2 * j) * MT + mt][lane], u = red[0][(2 * j + 1) * MT + mt][lane];
#pragma unroll
          for (int w = 1; w < WPB; ++w) {
            const float4 a = red[w][(2 * j) * MT + mt][lane], b = red[w][(2 * j + 1) * MT + mt][lane];
            g.x += a.x; g.y += a.y; g.z += a.z; g.w += a.w;
            u.x += b.x; u.y += b.y; u.z += b.z; u.w += b.w;
          }
          const float gv[4] = {g.x, g.y, g.z, g.w}, uv[4] = {u.x, u.y, u.z, u.w};
          const int n = ((tile0 + pass * kRedNT + 2 * j) >> 1) * kTileN + (lane & 15);
          if (n < sg.N) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int m = (mtile0 + mt) * 16 + 4 * (lane >> 4) + i;
              const float act = gv[i] / (1.0f + __expf(-gv[i]));       // silu
              if (m >= p.M) continue;
              const _Float16 h = static_cast<_Float16>(act * uv[i]);
              if (p.out_frag == 2) {
                // A fragment of the next layer: storage channel np of row m sits in k-step np / 32,
                // lane 16 ((np / 8) % 4) + m % 16, half np % 8
                const int np = next_pos[pass][it], mtile = mtile0 + mt;
                const int lane2 = 4 * (lane >> 4) + i + 16 * ((np >> 3) & 3);
                sg.out[(((static_cast<size_t>(mtile >> 2) * p.KS_out + (np >> 5)) * 4 + (mtile & 3)) * 64 + lane2) * 8 +
                       (np & 7)] = h;
              } else {
                sg.out[static_cast<int64_t>(m) * sg.ldo + n] = h;
              }
            }
          }
        }
      }
      return;
    }
  }

  // ---- sum the waves of this workgroup through LDS in wave order -----------------------
  constexpr int kSlots = kRedNT * MT;
  const size_t tile_id = static_cast<size_t>(chunk) * p.mgroups + mg;
  float4* my_part = p.part + ((tile_id * splits + split) * (kRedPasses * kSlots)) * 64 + lane;
#pragma unroll
  for (int pass = 0; pass < kRedPasses; ++pass) {
    if (pass > 0) __syncthreads();
#pragma unroll
    for (int nt = 0; nt < kRedNT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const floatx4 v = acc[pass * kRedNT + nt][mt];
        red[wave][nt * MT + mt][lane] = make_float4(v[0], v[1], v[2], v[3]);
      }
    __syncthreads();

    for (int slot = wave; slot < kSlots; slot += WPB) {
      float4 v = red[0][slot][lane];
#pragma unroll
      for (int w = 1; w < WPB; ++w) {
        const float4 o = red[w][slot][lane];
        v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
      }
      if (splits <= 1)
        store_fragment(p, v, mtile0 + slot % MT, tile0 + pass * kRedNT + slot / MT, lane);
      else
        store_device_scope(my_part + static_cast<size_t>(pass * kSlots + slot) * 64, v);
    }
  }
  if (splits <= 1) return;

  // ---- split launches: the workgroup that draws a tile's last ticket finishes the tile -----
  // Every wave's partial stores have completed (the barrier waits for each wave's outstanding
  // memory operations first) before one thread draws the ticket.  No workgroup waits for
  // another: all but the last one are done here.
  __shared__ unsigned ticket_lds;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's partial stores are done
  __syncthreads();
  if (threadIdx.x == 0)
    ticket_lds = __hip_atomic_fetch_add(p.tickets + tile_id, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (ticket_lds != static_cast<unsigned>(splits - 1)) return;
  if (threadIdx.x == 0)
    __hip_atomic_store(p.tickets + tile_id, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  constexpr int kAllSlots = kRedPasses * kSlots;
  constexpr int kPerWave = (kAllSlots + WPB - 1) / WPB;       // slots a wave finishes
  const float4* tile_part = p.part + (tile_id * splits * kAllSlots) * 64 + lane;
  // Every load below is unconditional (a split or slot past the end re-reads the last one and is
  // dropped by a select when added): loads under a branch end up next to their use, and the wave
  // would wait for each partial tile in turn instead of having them all in flight.
  float4 v[kPerWave];
#pragma unroll
  for (int i = 0; i < kPerWave; ++i) v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int sp0 = 0; sp0 < splits; sp0 += 4) {     // four partial tiles per slot in flight, added in split order
    float4 o[kPerWave][4];
#pragma unroll
    for (int i = 0; i < kPerWave; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int slot = wave + i * WPB < kAllSlots ? wave + i * WPB : kAllSlots - 1;
        const int sp = sp0 + j < splits ? sp0 + j : splits - 1;
        o[i][j] = load_device_scope(tile_part + (static_cast<size_t>(sp) * kAllSlots + slot) * 64);
      }
#pragma unroll
    for (int i = 0; i < kPerWave; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool use = sp0 + j < splits;
        v[i].x += use ? o[i][j].x : 0.f; v[i].y += use ? o[i][j].y : 0.f;
        v[i].z += use ? o[i][j].z : 0.f; v[i].w += use ? o[i][j].w : 0.f;
      }
  }
#pragma unroll
  for (int i = 0; i < kPerWave; ++i) {
    const int slot = wave + i * WPB;
    if (slot < kAllSlots) {
      const int pass = slot / kSlots, sl = slot - pass * kSlots;
      store_fragment(p, v[i], mtile0 + sl % MT, tile0 + pass * kRedNT + sl / MT, lane);
    }
  }
}

// xhat fragments from x by a column permutation (or identity): the prologue of
// the rotation-less layer and of the dense rotation.  Storage order keeps channels
// ascending inside the salient and inside the remaining part, so most 8-channel
// fragments are a run of consecutive channels: those are cut out of two aligned
// 16-byte loads; the others are gathered element by element.
__global__ __launch_bounds__(256) void gather_kernel(const _Float16* __restrict__ x, int64_t ldx,
                                                     int M, int KS, const int32_t* __restrict__ perm,
                                                     uint4* __restrict__ xf, int total,
                                                     unsigned* __restrict__ zero_ptr, int zero_count) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  // tickets of the GEMM launches that follow in this call, spread over the launch's threads
  for (int i = idx; i < zero_count; i += gridDim.x * 256) zero_ptr[i] = 0u;
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
      const int4 pa = *reinterpret_cast<const int4*>(perm + p0);
      const int4 pb = *reinterpret_cast<const int4*>(perm + p0 + 4);
      if (pb.w - pa.x == 7) {
        const int base = pa.x & ~7, sh = pa.x & 7;
        const uint4 lo = *reinterpret_cast<const uint4*>(row + base);
        uint4 hi = make_uint4(0, 0, 0, 0);
        if (sh) hi = *reinterpret_cast<const uint4*>(row + base + 8);   // sh > 0: the run reaches into it
        const uint32_t w[9] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w, 0u};
        uint32_t o[4] = {0, 0, 0, 0};
#pragma unroll
        for (int s2 = 0; s2 < 4; ++s2) {
          if ((sh >> 1) == s2) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
              o[k] = (sh & 1) ? __builtin_amdgcn_alignbyte(w[k + s2 + 1], w[k + s2], 2) : w[k + s2];
          }
        }
        v = make_uint4(o[0], o[1], o[2], o[3]);
      } else {
        const int c[8] = {pa.x, pa.y, pa.z, pa.w, pb.x, pb.y, pb.z, pb.w};
        uint16_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = __builtin_bit_cast(uint16_t, row[c[e]]);
        v.x = h[0] | (uint32_t(h[1]) << 16); v.y = h[2] | (uint32_t(h[3]) << 16);
        v.z = h[4] | (uint32_t(h[5]) << 16); v.w = h[6] | (uint32_t(h[7]) << 16);
      }
    }
  }
  xf[idx] = v;
}

// Head-wise rotation (Eq. 6): xhat_h = x_h fp16(Q_h).  One workgroup per (head,
// 16-channel column tile, 64-row block): wave w owns row tile w, issues every load
// it needs at once (x, Q_h fragments, storage positions), runs 4 MFMAs and scatters
// the tile to the storage position of each rotated channel.
__global__ __launch_bounds__(256) void rotate_headwise_kernel(
    const _Float16* __restrict__ x, int64_t ldx, int M, int KS, int H, const uint4* __restrict__ qh,
    const int32_t* __restrict__ pos, _Float16* __restrict__ xf, unsigned* __restrict__ zero_ptr,
    int zero_count) {
  // tickets of the GEMM launch that follows in this call, spread over the launch's threads
  for (int i = (blockIdx.y * gridDim.x + blockIdx.x) * 256 + threadIdx.x; i < zero_count;
       i += gridDim.x * gridDim.y * 256)
    zero_ptr[i] = 0u;
  const int lane = threadIdx.x & 63;
  const int mt = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // the eight column tiles of a head share x_h: keep them on one XCD (id % 8)
  const int h = (blockIdx.x & 7) + 8 * (blockIdx.x >> 6), ct = (blockIdx.x >> 3) & 7, mb = blockIdx.y;
  if (h >= H) return;
  const int m = mb * kMBlock + mt * 16 + (lane & 15);
  uint4 a[4], b[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    a[t] = make_uint4(0, 0, 0, 0);
    if (m < M)
      a[t] = *reinterpret_cast<const uint4*>(x + static_cast<int64_t>(m) * ldx + h * kHeadDim +
                                             t * kKStep + (lane >> 4) * 8);
    b[t] = qh[((static_cast<size_t>(h) * 8 + ct) * 4 + t) * 64 + lane];
  }
  const int p = pos[h * kHeadDim + ct * 16 + (lane & 15)];
  floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < 4; ++t) acc = mfma16(as_h8(a[t]), as_h8(b[t]), acc);
  const int ks = p >> 5, j = (p >> 3) & 3, e = p & 7;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int lane2 = 4 * (lane >> 4) + i + 16 * j;
    xf[(((static_cast<size_t>(mb) * KS + ks) * 4 + mt) * 64 + lane2) * 8 + e] =
        static_cast<_Float16>(acc[i]);
  }
}

// Measurement aid: a pure read stream.  Every wave reads `w_kib` KiB of its own from
// `src` (1 KiB per load, eight loads in flight) and then `x_kib` KiB from a buffer
// shared by all workgroups, and keeps nothing.  It shows what the memory system
// delivers for a launch of the GEMM's size and shape, with no arithmetic at all.
__global__ __launch_bounds__(1024) void stream_probe_kernel(const uint4* __restrict__ src,
                                                            const uint4* __restrict__ shared,
                                                            int w_kib, int x_kib, int shared_kib,
                                                            uint4* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const size_t gw = static_cast<size_t>(blockIdx.x) * (blockDim.x >> 6) + (threadIdx.x >> 6);
  uint4 acc = make_uint4(0, 0, 0, 0);
  const uint4* wp = src + gw * w_kib * 64 + lane;
  for (int i = 0; i < w_kib; i += 8) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      v[u] = i + u < w_kib ? wp[static_cast<size_t>(i + u) * 64] : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < 8; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
  }
  const int start = shared_kib ? static_cast<int>((threadIdx.x >> 6) * x_kib % shared_kib) : 0;
  for (int i = 0; i < x_kib; i += 8) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      int c = start + i + u;
      if (c >= shared_kib) c -= shared_kib;
      v[u] = i + u < x_kib ? shared[static_cast<size_t>(c) * 64 + lane] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
  }
  // never true for the probe's fill patterns; keeps the loads alive
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[gw * 64 + lane] = acc;
}

// ---- offline step on the device: What = W Q in fp64, one rounding to fp16 (Eq. 1) -----
// out[n][c] = fp16( sum_k W[n][k] * Q[k][c] ), W fp16 [N x D], fp64 FMA chain in increasing k.
// Q fp32: dense [D x D], or (headwise) blocks [D/128][128][128] of a block-diagonal rotation,
// where the sum runs over the 128 channels of c's head only (Eq. 5-6).
// 64 x 64 outputs per workgroup, 4 x 4 per thread, 16-deep LDS tiles.
__global__ __launch_bounds__(256) void rotate_weights_f64_kernel(const _Float16* __restrict__ W,
                                                                 const float* __restrict__ Q,
                                                                 uint16_t* __restrict__ out, int N,
                                                                 int D, int headwise) {
  __shared__ double sa[16][64 + 1];   // [k][row]
  __shared__ double sb[16][64];       // [k][col]
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int n0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int kb = headwise ? (c0 / kHeadDim) * kHeadDim : 0;      // first channel of the sum
  const int ke = headwise ? kb + kHeadDim : D;
  double acc[4][4] = {};
  for (int k0 = kb; k0 < ke; k0 += 16) {
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      const int r = i >> 4, k = i & 15;
      const int n = n0 + r;
      sa[k][r] = n < N ? static_cast<double>(W[static_cast<size_t>(n) * D + k0 + k]) : 0.0;
      const int kk = i >> 6, c = i & 63;
      const size_t qi = headwise ? (static_cast<size_t>(kb) + (k0 + kk - kb)) * kHeadDim + (c0 + c - kb)
                                 : static_cast<size_t>(k0 + kk) * D + c0 + c;
      sb[kk][c] = static_cast<double>(Q[qi]);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      double a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sa[k][ty * 4 + i]; b[i] = sb[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fma(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int n = n0 + ty * 4 + i;
    if (n >= N) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      out[static_cast<size_t>(n) * D + c0 + tx * 4 + j] = f64_to_f16_bits(acc[i][j]);
  }
}

// ---- launchers ------------------------------------------------------------------
static int hip_fail(hipError_t e, const char* what) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  return ROSAQ_ERR_HIP;
}

template <int BITS, int MT, int NT, int WPB, int DEPTH>
static int launch_gemm_t(const GemmDev& d, hipStream_t st) {
  const int xblocks = map_grid(d.chunks, d.mgroups) * (d.splits > 1 ? d.splits : 1);
  hipLaunchKernelGGL((gemm_kernel<BITS, MT, NT, WPB, DEPTH>), dim3(xblocks), dim3(WPB * 64), 0, st, d);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? ROSAQ_OK : hip_fail(e, "gemm_kernel launch");
}

// Tile choice.  At M = 64 the three per-CU resources are of the same order: vector
// memory inflow (about 120 GB/s per CU measured: the rotated activations of the
// tile's rows plus the tile's weights), VALU dequantisation (once per tile, so row
// splitting repeats it) and MFMA.  The model below prices a tile by
// max(inflow, VALU + MFMA) and the launch by the number of rounds of 256 tiles.
size_t gemm_part_bytes(const GemmShape& s, int M, int ntiles) {
  if (s.splits <= 1) return 0;
  const size_t chunks = (ntiles + s.nt - 1) / s.nt, mgroups = ((M + 15) / 16 + s.mt - 1) / s.mt;
  return chunks * mgroups * s.splits * (static_cast<size_t>(s.mt) * s.nt) * 1024;
}

// registers cap the units a wave can keep in flight
static int clamp_depth(int mt, int nt, int wpb, int depth) {
  int max_depth = 4;
  if (wpb == 4) {
    if (mt * nt == 16) max_depth = 3;
  } else if (wpb == 8) {
    if (mt * nt == 16) max_depth = 1;
    else if (mt == 4) max_depth = 2;
    else if (mt * nt == 8) max_depth = 3;
  } else {
    if (mt == 2) max_depth = 2;
    else if (nt == 2) max_depth = 3;
  }
  return std::min(depth, max_depth);
}

static GemmShape pick_unsplit(int M, int ntiles, int D, int bits, const GemmTune& tune);

// Split-K across workgroups (launches of up to 64 rows).  Measured on the 7B / 13B shapes at
// M = 64, a split launch loses wherever the unsplit one already fills the chip: a 4096 x 4096 layer
// takes 8.6 us as 256 tiles of 32 x 32 and 12.4 us as 64 tiles of 64 x 64 cut in 2, 3 or 4, because
// the partial tiles, the ticket and the last workgroup's pass over the partials follow one
// another at the end of a launch that is already bound by latency, not by bytes.  It wins where
// whole 64-row tiles leave compute units idle over a long contraction: 13824 -> 5120 runs as
// 160 workgroups of 32 x 64 in 25.9 us, as 80 x 3 workgroups of 64 x 64 in 22.4 us.  The default
// therefore splits only such launches; rosaq_tune("splits", n) forces any count for tests.
GemmShape pick_gemm_shape(int M, int ntiles, int D, int bits, const GemmTune& tune, size_t part_bytes,
                          int ticket_count, int ks_s) {
  GemmShape base = pick_unsplit(M, ntiles, D, bits, tune);
  base.splits = 1;
  const int mtiles = (M + 15) / 16;
  if (tune.splits == 1 || part_bytes == 0 || ticket_count <= 0 || mtiles > 4) return base;
  (void)ks_s;
  const int mt = mtiles > 2 ? 4 : mtiles;                           // all rows in one workgroup
  auto candidate = [&](int nt, int sp) {
    GemmShape c{mt, nt, 8, 1, sp};
    if (mt == 4 && nt == 6) c.wpb = 4;
    c.depth = clamp_depth(c.mt, c.nt, c.wpb, tune.depth >= 1 ? tune.depth : 2);
    if (nt == 3 || nt == 6) {
      const int cap = mt == 4 ? 1 : (nt == 6 ? 2 : 3);
      c.depth = std::min(tune.depth >= 1 ? tune.depth : (nt == 6 ? 1 : cap), cap);
    }
    if (bits == 16) {
      const int per_unit = 16 * (c.mt + c.nt);
      c.depth = tune.depth >= 1 && tune.depth <= 4 ? tune.depth : 3;
      while (c.depth > 1 && c.depth * per_unit + 4 * c.mt * c.nt > 232) --c.depth;
    }
    return c;
  };
  auto fits = [&](const GemmShape& c) {
    const int tiles = ((ntiles + c.nt - 1) / c.nt) * ((mtiles + c.mt - 1) / c.mt);
    return tiles <= ticket_count && gemm_part_bytes(c, M, ntiles) <= part_bytes;
  };
  if (tune.splits > 1) {                                            // forced: tests and measurements
    int nt = tune.nt ? tune.nt : 4;
    if ((nt == 3 || nt == 6) && (mt < 2 || (bits == 16 && nt == 6))) nt = 4;
    if (nt != 1 && nt != 2 && nt != 3 && nt != 4 && nt != 6) nt = 4;
    if (bits == 16 && mt == 1 && nt == 3) nt = 4;
    const GemmShape c = candidate(nt, tune.splits);
    return fits(c) ? c : base;
  }
  const int unsplit_wgs = ((ntiles + base.nt - 1) / base.nt) * ((mtiles + base.mt - 1) / base.mt);
  const int chunks = (ntiles + 3) / 4;
  const int sp = std::min(4, 256 / std::max(chunks, 1));
  if (bits != 16 && mtiles >= 3 && D >= 8192 && unsplit_wgs <= 192 && sp >= 2) {
    const GemmShape c = candidate(4, sp);
    if (fits(c)) return c;
  }
  return base;
}

static GemmShape pick_unsplit(int M, int ntiles, int D, int bits, const GemmTune& tune) {
  GemmShape s;
  const int mtiles = (M + 15) / 16;
  const double k = static_cast<double>(D);
  const double wbytes = bits == 16 ? 2.0 : (bits == 3 ? 0.46 : 0.58);   // per weight incl. scale / zero
  double best = 1e30;
  s.mt = s.nt = 1;
  for (int mt = 1; mt <= 4; mt <<= 1) {
    if (mt > 1 && mt / 2 >= mtiles) break;           // do not pad rows beyond the next tile size
    for (int nt = 1; nt <= 4; nt <<= 1) {
      const double tiles = static_cast<double>((ntiles + nt - 1) / nt) * ((mtiles + mt - 1) / mt);
      const double rounds = std::ceil(tiles / 256.0);
      const double inflow = (mt * 16 * k * 2.0 + nt * 16 * k * wbytes) / 120e3;
      const double valu = bits == 16 ? 0.0 : nt * k * (bits == 3 ? 2.9e-4 : 1.7e-4) + mt * nt * k * 1.3e-5;
      const double mfma = mt * nt * k * 5.2e-5;
      const double t = rounds * std::max(inflow, valu + mfma);
      if (t < best * 0.999) { best = t; s.mt = mt; s.nt = nt; }
    }
  }
  // 32 x 96 and 64 x 48 tiles against the shape chosen above.  Measured launch times of the
  // low-bit kernels at 32 to 256 rows order like rounds x (inflow + VALU issue) per workgroup:
  // the bytes it pulls through its CU's vector-memory path at 128 GB/s (its rows of the rotated
  // activations plus its weights) plus the four cycles per wave64 VALU instruction of its two
  // waves per SIMD (9 instructions per 8 weights to convert, 4 per output fragment and group
  // to scale, 40 per group otherwise).  q/k/v of a 7B attention block in one launch at M = 64:
  // 192 workgroups of 64 x 64 take 16.2 us, 256 of 32 x 96 15.0, 256 of 64 x 48 14.5; gate + up
  // of a 7B MLP 28.7 / 26.9 / 26.3 us, at M = 32 32 x 96 tiles make it one round (19.7 -> 16.2).
  // Eight waves like every default shape: the summation order stays the same.
  if (bits != 16 && mtiles >= 2) {
    const double groups = k / 128.0;
    auto cost = [&](int mt, int nt) {
      const int wgs = ((ntiles + nt - 1) / nt) * ((mtiles + mt - 1) / mt);
      const double inflow = (mt * 32.0 + nt * 16 * wbytes) * k / 128e3;
      const double valu = (nt * ((bits == 3 ? 40 : 36) + 4 * mt) + 40) * (groups / 8) * 8 / 2000.0;
      return ((wgs + 255) / 256) * (inflow + valu);
    };
    double best_alt = cost(s.mt, s.nt) * 0.97;   // a change has to promise 3 %
    const int mt0 = s.mt, nt0 = s.nt;
    if (mt0 * nt0 >= 4) {
      if (cost(2, 6) < best_alt) { best_alt = cost(2, 6); s.mt = 2; s.nt = 6; }
      if (mtiles >= 3 && cost(4, 3) < best_alt) { best_alt = cost(4, 3); s.mt = 4; s.nt = 3; }
    }
  }
  // The same for all-fp16 layers (the dense rotation), which have no conversion: 48-channel tiles
  // by rounds x inflow.  A 5120 x 5120 rotation at M = 64 is 160 workgroups of 32 x 64 but 214 of
  // 32 x 48 (24.3 -> 21.7 us); 11008 x 11008 is 172 of 64 x 64 but 230 of 64 x 48 (64.6 -> 60.0 us).
  if (bits == 16 && mtiles >= 2 && s.mt * s.nt >= 4) {
    auto cost = [&](int mt, int nt) {
      const int wgs = ((ntiles + nt - 1) / nt) * ((mtiles + mt - 1) / mt);
      return ((wgs + 255) / 256) * static_cast<double>(mt + nt);
    };
    double best_alt = cost(s.mt, s.nt) * 0.97;
    if (cost(2, 3) < best_alt) { best_alt = cost(2, 3); s.mt = 2; s.nt = 3; }
    if (mtiles >= 3 && cost(4, 3) < best_alt) { s.mt = 4; s.nt = 3; }
  }
  if (tune.mt == 1 || tune.mt == 2 || tune.mt == 4) s.mt = tune.mt;
  if (tune.nt == 1 || tune.nt == 2 || tune.nt == 4) s.nt = tune.nt;
  if ((tune.nt == 3 || tune.nt == 6) && bits != 16 && s.mt >= 2) s.nt = tune.nt;
  if (tune.nt == 3 && bits == 16 && s.mt >= 2) s.nt = 3;
  s.wpb = 8;
  if (tune.wpb == 16 && s.mt * s.nt <= 2) s.wpb = 16;   // 16 waves leave 128 registers per lane
  // a single 16 x 16 tile per workgroup (decode steps of a few rows): sixteen waves with one
  // unit in flight each beat eight waves with two (8.3 against 9.3 us for 11008 -> 4096 at M = 1)
  const bool skinny16 = tune.wpb == 0 && tune.depth == 0 && bits != 16 && s.mt == 1 && s.nt == 1;
  if (skinny16) s.wpb = 16;
  if (tune.wpb == 4 && s.mt * s.nt >= 8) s.wpb = 4;     // one wave per SIMD: 512 registers
  // loads in flight per wave: depth 1 variants of the small tiles fit 128 registers,
  // so two workgroups share a CU and cover each other's latency
  s.depth = ((s.mt * s.nt <= 4 && s.mt > 1) || s.mt * s.nt == 16) ? 1 : 2;   // skinny tiles: latency, not occupancy
  if (tune.depth >= 1 && tune.depth <= 4) s.depth = tune.depth;
  if (skinny16) s.depth = 1;
  // two tiles per workgroup at a single row tile, in a launch that does not fill one round of
  // 256 workgroups: sixteen waves with two units in flight (13824 -> 5120 at M = 1: 160
  // workgroups, 13.5 against 14.9 us with eight waves; launches of several rounds lose 15-25 %)
  const bool skinny16x2 = tune.wpb == 0 && tune.depth == 0 && bits != 16 && s.mt == 1 && s.nt == 2 &&
                          (ntiles + 1) / 2 * mtiles <= 256;
  if (skinny16x2) { s.wpb = 16; s.depth = 2; }
  // deepest prefetch that still fits the register file without spilling
  int max_depth = 4;
  if (s.wpb == 4) {
    if (s.mt * s.nt == 16) max_depth = 3;
  } else if (s.wpb == 8) {
    if (s.mt * s.nt == 16) max_depth = 1;
    else if (s.mt == 4) max_depth = 2;
    else if (s.mt * s.nt == 8) max_depth = 3;
  } else {
    if (s.mt == 2) max_depth = 2;
    else if (s.nt == 2) max_depth = 3;
  }
  s.depth = std::min(s.depth, max_depth);
  if (s.depth == 1 && s.mt * s.nt > 4 && s.mt * s.nt < 16) s.depth = 2;
  if (s.nt == 3 || s.nt == 6) {
    // 48- and 96-channel tiles (they make 768- and 1376-tile launches fit one round of 256)
    if (s.mt == 4 && s.nt == 6) {
      s.wpb = 4;                                        // 96 accumulator registers: one wave per SIMD
      s.depth = 1;
    } else {
      s.wpb = 8;
      const int cap = s.mt == 4 ? 1 : (s.nt == 6 ? 2 : 3);
      s.depth = std::min(tune.depth >= 1 ? tune.depth : (s.nt == 6 ? 1 : cap), cap);
    }
  }
  if (bits == 16) {
    // all-fp16 layers: a unit is four k-steps, 16 * (mt + nt) registers per unit in flight
    s.wpb = 8;
    const int per_unit = 16 * (s.mt + s.nt);
    s.depth = tune.depth >= 1 && tune.depth <= 4 ? tune.depth : 3;
    while (s.depth > 1 && s.depth * per_unit + 4 * s.mt * s.nt > 232) --s.depth;
  }
  return s;
}

// 0 = launched, 1 = no kernel is instantiated for this shape, negative = error
static int launch_gemm_shape(const GemmArgs& a, const GemmShape& sh, void* stream) {
  GemmDev d;
  d.xf = static_cast<const uint4*>(a.xf);
  d.xrow = static_cast<const _Float16*>(a.xrow);
  d.ldx = a.ldx;
  d.M = a.M; d.ks_s = a.ks_s; d.G = a.G; d.KS = a.KS; d.KS_out = a.KS_out;
  d.out_frag = a.out_frag;
  d.out_pos = static_cast<const int*>(a.out_pos);
  d.nseg = a.nseg;
  int tiles = 0;   // valid channel tiles of all layers, in launch order
  for (int i = 0; i < kMaxBatch; ++i) {
    const GemmSegArgs& sa = a.seg[i < a.nseg ? i : 0];
    if (i < a.nseg) tiles += (sa.N + kTileN - 1) / kTileN;
    d.seg[i].wS = static_cast<const uint4*>(sa.wS);
    d.seg[i].wq = static_cast<const uint32_t*>(sa.wq);
    d.seg[i].out = static_cast<_Float16*>(sa.out);
    d.seg[i].ldo = sa.ldo;
    d.seg[i].N = sa.N;
    d.seg[i].tile_end = tiles;
  }
  if (a.swiglu && (sh.nt & 1)) return 1;   // pairs of tiles need an even tile count per workgroup
  d.chunks = (tiles + sh.nt - 1) / sh.nt;
  d.mgroups = ((a.M + 15) / 16 + sh.mt - 1) / sh.mt;
  d.splits = a.swiglu ? 1 : sh.splits;
  d.part = static_cast<float4*>(a.part);
  d.tickets = static_cast<unsigned*>(a.tickets);
  d.zero_ptr = static_cast<unsigned*>(a.zero_ptr);
  d.zero_count = a.zero_count;
  d.swiglu = a.swiglu;
  const int bits = a.G == 0 ? 16 : a.bits;
  hipStream_t st = static_cast<hipStream_t>(stream);
#define ROSAQ_CASE(B, MT_, NT_, W)                                              \
  if (bits == B && sh.mt == MT_ && sh.nt == NT_ && sh.wpb == W) {              \
    if (sh.depth == 1) return launch_gemm_t<B, MT_, NT_, W, 1>(d, st);           \
    if (sh.depth == 2) return launch_gemm_t<B, MT_, NT_, W, 2>(d, st);           \
    if (sh.depth == 3) return launch_gemm_t<B, MT_, NT_, W, 3>(d, st);           \
    return launch_gemm_t<B, MT_, NT_, W, 4>(d, st);                              \
  }
#define ROSAQ_CASES(B)                                                          \
  ROSAQ_CASE(B, 1, 1, 8) ROSAQ_CASE(B, 1, 2, 8) ROSAQ_CASE(B, 1, 4, 8)          \
  ROSAQ_CASE(B, 2, 1, 8) ROSAQ_CASE(B, 2, 2, 8) ROSAQ_CASE(B, 2, 4, 8)          \
  ROSAQ_CASE(B, 4, 1, 8) ROSAQ_CASE(B, 4, 2, 8) ROSAQ_CASE(B, 4, 4, 8)          \
  ROSAQ_CASE(B, 4, 4, 4) ROSAQ_CASE(B, 4, 2, 4) ROSAQ_CASE(B, 2, 4, 4)          \
  ROSAQ_CASE(B, 1, 1, 16) ROSAQ_CASE(B, 1, 2, 16) ROSAQ_CASE(B, 2, 1, 16)
  ROSAQ_CASES(4)
  ROSAQ_CASES(3)
  ROSAQ_CASES(16)
#define ROSAQ_WIDE(B) ROSAQ_CASE(B, 4, 3, 8) ROSAQ_CASE(B, 2, 3, 8) ROSAQ_CASE(B, 2, 6, 8) ROSAQ_CASE(B, 4, 6, 4)
  ROSAQ_WIDE(4)
  ROSAQ_WIDE(3)
  ROSAQ_CASE(16, 2, 3, 8) ROSAQ_CASE(16, 4, 3, 8)
#undef ROSAQ_WIDE
#undef ROSAQ_CASES
#undef ROSAQ_CASE
  return 1;
}

int launch_gemm(const GemmArgs& a, const GemmTune& tune, void* stream) {
  int tiles_total = 0;
  for (int i = 0; i < a.nseg; ++i) tiles_total += (a.seg[i].N + kTileN - 1) / kTileN;
  const int bits = a.G == 0 ? 16 : a.bits;
  auto shape = [&](const GemmTune& t) {
    return pick_gemm_shape(a.M, tiles_total, a.KS * kKStep, bits, t, a.part ? a.part_bytes : 0,
                           a.tickets ? a.ticket_count : 0, a.ks_s);
  };
  GemmTune t0 = tune;
  if (a.swiglu) {
    // a gated pair runs unsplit with an even number of channel tiles per workgroup
    t0.splits = 1;
    const GemmShape s0 = shape(t0);
    // 48-channel tiles become 32 x 96 ones (gate + up of a 7B MLP at M = 64: 26.9 us against 28.7 us
    // as 64 x 64 tiles, which need a second round of workgroups)
    if (s0.nt == 3) { t0.nt = 6; t0.mt = 2; }
    else if (s0.nt & 1) t0.nt = 2;
  }
  int rc = launch_gemm_shape(a, shape(t0), stream);
  // a forced combination that no kernel is built for falls back to the heuristic's choice
  if (rc == 1) {
    GemmTune t1{};
    if (a.swiglu) {
      t1.splits = 1;
      const GemmShape s1 = shape(t1);
      if (s1.nt == 3) { t1.nt = 6; t1.mt = 2; }
      else if (s1.nt & 1) t1.nt = 2;
    }
    rc = launch_gemm_shape(a, shape(t1), stream);
  }
  if (rc == 1) {
    set_error("no kernel for this bits / tile combination");
    return ROSAQ_ERR_ARG;
  }
  return rc;
}

int launch_rotate_weights_f64(const void* W_dev, const void* Q_dev, void* out_dev, int N, int D,
                              int headwise, void* stream) {
  hipLaunchKernelGGL(rotate_weights_f64_kernel, dim3(D / 64, (N + 63) / 64), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const _Float16*>(W_dev),
                     static_cast<const float*>(Q_dev), static_cast<uint16_t*>(out_dev), N, D, headwise);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? ROSAQ_OK : hip_fail(e, "rotate_weights_f64_kernel launch");
}

int launch_stream_probe(const void* src, const void* shared, int workgroups, int threads, int w_kib,
                        int x_kib, int shared_kib, void* sink, void* stream) {
  hipLaunchKernelGGL(stream_probe_kernel, dim3(workgroups), dim3(threads), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(src),
                     static_cast<const uint4*>(shared), w_kib, x_kib, shared_kib,
                     static_cast<uint4*>(sink));
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? ROSAQ_OK : hip_fail(e, "stream_probe_kernel launch");
}

int launch_gather(const void* x, int64_t ldx, int M, int D, const int32_t* perm_dev, void* xf,
                  void* zero_ptr, int zero_count, void* stream) {
  const int KS = D / kKStep, mblocks = (M + kMBlock - 1) / kMBlock;
  const int total = mblocks * KS * 256;
  hipLaunchKernelGGL(gather_kernel, dim3((total + 255) / 256), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const _Float16*>(x), ldx, M, KS,
                     perm_dev, static_cast<uint4*>(xf), total, static_cast<unsigned*>(zero_ptr), zero_count);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? ROSAQ_OK : hip_fail(e, "gather_kernel launch");
}

int launch_rotate_headwise(const void* x, int64_t ldx, int M, int D, const void* qh,
                           const int32_t* pos_dev, void* xf, void* zero_ptr, int zero_count,
                           void* stream) {
  const int H = D / kHeadDim, mblocks = (M + kMBlock - 1) / kMBlock;
  hipLaunchKernelGGL(rotate_headwise_kernel, dim3(((H + 7) / 8) * 64, mblocks), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const _Float16*>(x), ldx, M,
                     D / kKStep, H, static_cast<const uint4*>(qh), pos_dev,
                     static_cast<_Float16*>(xf), static_cast<unsigned*>(zero_ptr), zero_count);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? ROSAQ_OK : hip_fail(e, "rotate_headwise_kernel launch");
}

}  // namespace rosaq
