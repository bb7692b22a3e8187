// Internal declarations shared by the host packer, the C ABI and the kernel launchers.
#pragma once
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "rosaq.h"

namespace rosaq {

constexpr int kGroup = 128;    // quantisation group (Sec. 3.3: groups of 128 channels)
constexpr int kHeadDim = 128;  // block size of the head-wise rotation (Eq. 6)
constexpr int kKStep = 32;     // contraction depth of one v_mfma_f32_16x16x32_f16
constexpr int kTileN = 16;     // output channels per MFMA tile
constexpr int kMBlock = 64;    // rows of x handled by one workgroup pass (4 MFMA row tiles)

// ---- fp16 <-> fp64 on the host (rosaq_pack.cpp) -------------------------------
uint16_t f64_to_f16(double v);  // round-half-to-even, one rounding, overflow -> inf
double f16_to_f64(uint16_t h);

// Host-side result of the offline step (Eq. 3): canonical arrays in storage order.
struct Canonical {
  int N = 0, D = 0, K = 0, bits = 0, q_mode = 0;
  int G = 0;                          // low-bit groups per output row, (D-K)/128
  std::vector<int32_t> salient_idx;   // [K] ascending
  std::vector<int32_t> perm;          // [D] storage position -> rotated channel
  std::vector<int32_t> pos;           // [D] rotated channel -> storage position
  std::vector<uint16_t> W_S;          // [N x K] fp16
  std::vector<uint8_t> codes;         // [N x (D-K)]
  std::vector<uint16_t> scales;       // [N x G] fp16
  std::vector<uint16_t> zeros;        // [N x G] fp16 (integer valued)
};

// Pieces of the offline step that also serve the device path: input checks, and the salient set
// with the storage order (fills the shape fields, salient_idx, perm, pos).
int pack_validate(const rosaq_pack_desc& d, std::string* err);
void pack_select(const rosaq_pack_desc& d, Canonical* c);

// Sec. 3.1-3.3 on the host.  Returns ROSAQ_OK or an error code with `err` filled.
// `rotated16` (optional): What = fp16(W Q) [N x D] already computed elsewhere (the device path).
int pack_host(const rosaq_pack_desc& d, Canonical* out, std::string* err,
              const std::vector<uint16_t>* rotated16 = nullptr);

// Device images (host staging copies) in the kernels' fragment order.
struct DeviceImage {
  std::vector<uint32_t> wS;   // [ntiles][K/32][64 lanes][4 dwords]   fp16 salient fragments
  // records [ntiles][G]: int4 [64][4] codes, int3 [64][3] codes, then [16] scale | zero << 16
  std::vector<uint32_t> wq;
  std::vector<uint32_t> sz;   // staging only (merged into wq)
  std::vector<uint32_t> qf;   // FULL: [D/16][D/32][64][4]; HEADWISE: [H][8][4][64][4]; fp16(Q)
};
void build_device_image(const Canonical& c, const float* Q, DeviceImage* img);

// ---- kernel launchers (rosaq_kernels.hip) -------------------------------------
constexpr int kMaxBatch = 4;   // layers per launch that share one rotated input
struct GemmSegArgs {
  const void* wS;        // fp16 fragments  [ntiles][ks_s][64]   x 16 B
  const void* wq;        // low-bit records: code fragment + scale/zero words
  void* out;             // y (row-major fp16) or xhat fragments
  int64_t ldo;           // leading dimension of y
  int N;                 // valid output channels
};
struct GemmArgs {
  const void* xf;        // xhat fragments  [mblocks][KS][4][64] x 16 B
  const void* xrow;      // or (all-fp16 launches with ks_s % 4 == 0): row-major fp16 x, stride ldx
  int64_t ldx;
  GemmSegArgs seg[kMaxBatch];
  int nseg;
  int M;                 // valid rows
  int ks_s;              // fp16 k-steps (K/32)
  int G;                 // low-bit groups
  int KS;                // k-steps of the xf operand (D/32)
  int KS_out;            // k-steps of the output when out is in fragment order
  int bits;              // 3 or 4 (ignored when G == 0)
  int out_frag;          // 0: y row-major, 1: xhat fragment order, 2 (gated pair only): input
                         // fragments of a following layer, channel n at storage position out_pos[n]
  const void* out_pos = nullptr;   // device int32 [N] for out_frag == 2
  // split-K across workgroups (optional): room for fp32 partial tiles and tile tickets.  A launch
  // is split only if both fit; tickets must be zero before the launch and are zero after it.
  void* part = nullptr;
  size_t part_bytes = 0;
  void* tickets = nullptr;
  int ticket_count = 0;
  void* zero_ptr = nullptr;   // 32-bit words this launch clears for a later launch of the call
  int zero_count = 0;
  int swiglu = 0;             // nseg == 2 layers of equal N: store silu(seg 0) * seg 1 to seg[0].out
};
constexpr int kMaxSplits = 16;
constexpr int kTicketsPerLaunch = 4096;   // ticket words per GEMM launch kept in the workspace
struct GemmTune { int mt = 0, nt = 0, wpb = 0, depth = 0, splits = 0; };   // 0 = heuristic
struct GemmShape { int mt, nt, wpb, depth, splits; };
// `part_bytes` / `ticket_count`: what the caller can offer for split-K (0 = never split)
GemmShape pick_gemm_shape(int M, int ntiles, int D, int bits, const GemmTune& tune,
                          size_t part_bytes = 0, int ticket_count = 0, int ks_s = -1);
// bytes of partial tiles a launch of this shape needs
size_t gemm_part_bytes(const GemmShape& s, int M, int ntiles);
int launch_gemm(const GemmArgs& a, const GemmTune& tune, void* stream);
// Host copy of the kernel's workgroup -> (channel chunk, row group) map: b < 0 returns the grid
// size, otherwise 1 and the pair, or 0 for a padding workgroup that exits at once.
int block_map_host(int b, int chunks, int mgroups, int* chunk, int* mg);
// both prologue launchers also clear `zero_count` 32-bit words at `zero_ptr` (the tickets of the
// GEMM launches that follow in the same call)
int launch_gather(const void* x, int64_t ldx, int M, int D, const int32_t* perm_dev,
                  void* xf, void* zero_ptr, int zero_count, void* stream);
int launch_rotate_headwise(const void* x, int64_t ldx, int M, int D, const void* qh,
                           const int32_t* pos_dev, void* xf, void* zero_ptr, int zero_count,
                           void* stream);

// Dense rotation of up to 64 rows as slabs of the contraction plus a summing launch
// (rosaq_rotate.hip).  pick_rotate_slabs: `forced` if slabs of that count fit the kernel, else 0;
// `part` needs rotate_slab_part_bytes(D, slabs) bytes.  The first launch also clears `zero_count`
// 32-bit words at `zero_ptr`.
int pick_rotate_slabs(int D, int forced);
size_t rotate_slab_part_bytes(int D, int slabs);
int launch_rotate_slabs(const void* x, int64_t ldx, int M, int D, const void* qf, int slabs, void* part,
                        void* xf_out, void* zero_ptr, int zero_count, void* stream);

int launch_rotate_weights_f64(const void* W_dev, const void* Q_dev, void* out_dev, int N, int D,
                              int headwise, void* stream);
int launch_stream_probe(const void* src, const void* shared, int workgroups, int threads, int w_kib,
                        int x_kib, int shared_kib, void* sink, void* stream);

// Offline step on the device (rosaq_quant.hip): What16 [N x D] fp16 (device) -> fragment images and
// canonical arrays (all device pointers; `flag` is one word that is set if What16 holds Inf / NaN).
struct QuantPackArgs {
  const void* what16;
  int N, D, K, bits;
  const int32_t* perm;   // [D] storage position -> rotated channel
  void* wS_image;        // [tiles][K/32][64] x 16 B
  void* wq_image;        // records [tiles][G]
  void* W_S;             // fp16 [N x K]
  void* codes;           // uint8 [N x (D-K)]
  void* scales;          // fp16 [N x G]
  void* zeros;           // fp16 [N x G]
  void* flag;
};
int launch_quantize_pack(const QuantPackArgs& a, void* stream);
int launch_rotation_image(const void* Q_dev, int D, int headwise, const int32_t* perm_dev, void* qf_image,
                          void* stream);

int pca_headwise_device(const void* X_dev, int n_cal, int D, int64_t ldx, float* Q_host,
                        double* eig_host, void* stream);
int pca_full_device(const void* X_dev, int n_cal, int D, int64_t ldx, float* Q_host, double* eig_host,
                    void* stream);

// Library-owned scratch (rosaq_static.hip): the device address of this GPU's copy of a fixed
// kStaticScratchBytes array, looked up once per device.
constexpr size_t kStaticScratchBytes = size_t{8} << 20;
int static_scratch(void** ptr_out);

void set_error(const std::string& s);

}  // namespace rosaq

struct rosaq_packed {
  rosaq::Canonical c;
  bool host_only = true;
  int device = -1;
  void* d_blob = nullptr;
  size_t blob_bytes = 0;
  // sub-buffers inside d_blob
  void* d_wS = nullptr;
  void* d_wq = nullptr;
  void* d_qf = nullptr;
  int32_t* d_perm = nullptr;
  int32_t* d_pos = nullptr;
  uint64_t rot_fingerprint = 0;   // hash of (q_mode, Q, storage order): equal => same xhat
};
