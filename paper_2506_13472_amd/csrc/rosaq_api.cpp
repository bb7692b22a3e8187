// C ABI of the library: argument validation, handle ownership, device upload and
// the per-call launch sequence.  No arithmetic of the method happens here.
#include <hip/hip_runtime_api.h>

#include <climits>
#include <cstdlib>
#include <cstring>
#include <exception>
#include <new>
#include <type_traits>

#include "rosaq_internal.h"

namespace rosaq {

static thread_local std::string g_error;
void set_error(const std::string& s) { g_error = s; }

static GemmTune g_tune;         // all zero = heuristics
static GemmTune g_tune_rot;     // same, for the dense-rotation launch
static int g_tune_stages = 3;  // bit 0: prologue kernels, bit 1: main GEMM (timing aid)

static int fail(int code, const std::string& msg) {
  set_error(msg);
  return code;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }


// Workspace carve-up for one call with M rows.
// [xhat fragments | second copy for the dense rotation | tickets of the rotation GEMM and of the
// main GEMM | fp32 partial tiles of split launches].  `required` is what a call cannot do without;
// whatever the caller gives beyond it is room for partial tiles.
struct WsPlan {
  size_t xf_a = 0, xf_b = 0, tickets = 0, part = 0, required = 0, total = 0;
};
constexpr size_t kTicketBytes = 2 * static_cast<size_t>(kTicketsPerLaunch) * sizeof(uint32_t);

// partial tiles of one launch at the largest split: rows padded to whole tiles, fp32
static size_t part_room(int M, size_t channels) {
  if (M > 64) return 0;                                   // only launches of up to 64 rows are split
  const size_t rows = M > 32 ? 64 : (M > 16 ? 32 : 16);
  return static_cast<size_t>(kMaxSplits) * rows * align_up(channels, 96) * 4;
}

static WsPlan plan_workspace(const rosaq_packed& p, int M, size_t channels_total = 0) {
  WsPlan w;
  const Canonical& c = p.c;
  const size_t mblocks = (static_cast<size_t>(M) + kMBlock - 1) / kMBlock;
  const size_t xf_bytes = mblocks * (c.D / kKStep) * 4 * 64 * 16;
  size_t off = 0;
  w.xf_a = off; off += align_up(xf_bytes, 256);
  if (c.q_mode == ROSAQ_Q_FULL) {
    w.xf_b = off; off += align_up(xf_bytes, 256);
  }
  w.tickets = off; off += kTicketBytes;
  w.required = off;
  w.part = off;
  const size_t widest = std::max<size_t>(channels_total ? channels_total : c.N,
                                         c.q_mode == ROSAQ_Q_FULL ? c.D : 0);
  off += align_up(part_room(M, widest), 256);
  w.total = off;
  return w;
}

static int check_desc(const rosaq_pack_desc* d) {
  if (!d) return fail(ROSAQ_ERR_NULL, "desc is NULL");
  if (!d->W) return fail(ROSAQ_ERR_NULL, "desc.W is NULL");
  if (!d->eigenvalues) return fail(ROSAQ_ERR_NULL, "desc.eigenvalues is NULL");
  if (d->q_mode < ROSAQ_Q_NONE || d->q_mode > ROSAQ_Q_HEADWISE)
    return fail(ROSAQ_ERR_ARG, "q_mode is not one of ROSAQ_Q_*");
  if (d->q_mode != ROSAQ_Q_NONE && !d->Q) return fail(ROSAQ_ERR_NULL, "desc.Q is NULL");
  if (d->bits != 3 && d->bits != 4) return fail(ROSAQ_ERR_ARG, "bits must be 3 or 4");
  if (d->group != kGroup) return fail(ROSAQ_ERR_ARG, "group must be 128");
  if (d->q_mode == ROSAQ_Q_HEADWISE && d->head_dim != kHeadDim)
    return fail(ROSAQ_ERR_ARG, "head_dim must be 128");
  if (d->select_rule < ROSAQ_SELECT_TOP || d->select_rule > ROSAQ_SELECT_TOP_AND_BOTTOM)
    return fail(ROSAQ_ERR_ARG, "select_rule is not one of ROSAQ_SELECT_*");
  if (d->out_features < 1 || d->in_features < 1)
    return fail(ROSAQ_ERR_SHAPE, "out_features and in_features must be positive");
  if (d->in_features % 128 != 0) return fail(ROSAQ_ERR_SHAPE, "in_features must be a multiple of 128");
  if (d->K < 0 || d->K > d->in_features) return fail(ROSAQ_ERR_SHAPE, "K must be in [0, in_features]");
  if (d->K % kKStep != 0) return fail(ROSAQ_ERR_SHAPE, "K must be a multiple of 32");
  if ((d->in_features - d->K) % d->group != 0)
    return fail(ROSAQ_ERR_SHAPE, "in_features - K must be a multiple of group");
  if (d->ldw < d->in_features) return fail(ROSAQ_ERR_SHAPE, "ldw is smaller than in_features");
  if (d->select_rule == ROSAQ_SELECT_TOP_PER_HEAD && d->K % (d->in_features / kHeadDim) != 0)
    return fail(ROSAQ_ERR_SHAPE, "K must be a multiple of the number of 128-channel heads");
  if (d->select_rule == ROSAQ_SELECT_TOP_AND_BOTTOM && d->K % 2 != 0)
    return fail(ROSAQ_ERR_SHAPE, "K must be even for TOP_AND_BOTTOM");
  if (d->select_rule == ROSAQ_SELECT_CONSECUTIVE &&
      (d->select_arg < 0 || d->select_arg > d->in_features - d->K))
    return fail(ROSAQ_ERR_SHAPE, "select_arg must lie in [0, in_features - K]");
  return ROSAQ_OK;
}

#define ROSAQ_HIP(call)                                                         \
  do {                                                                          \
    hipError_t e_ = (call);                                                     \
    if (e_ != hipSuccess) {                                                     \
      set_error(std::string(#call) + ": " + hipGetErrorString(e_));            \
      return ROSAQ_ERR_HIP;                                                     \
    }                                                                           \
  } while (0)

// The offline step with the layer on the GPU: upload W (and Q), rotate in fp64 (Eq. 1), then one
// pass from the rotated fp16 weight to the fragment images the kernels read and to the canonical
// arrays (Sec. 3.2-3.3, Eq. 3), which come back to the host for rosaq_packed_export.  Only the
// input checks and the ranking of D eigenvalues stay on the host.
static int pack_device(const rosaq_pack_desc& d, hipStream_t st, rosaq_packed* p) {
  std::string err;
  int rc = pack_validate(d, &err);
  if (rc != ROSAQ_OK) return fail(rc, err);
  pack_select(d, &p->c);
  Canonical& c = p->c;
  const size_t N = c.N, D = c.D, K = c.K, C = D - K, G = c.G;
  const size_t ntiles = (N + 127) / 128 * 8, ks_s = K / kKStep;
  const bool rotate = d.q_mode != ROSAQ_Q_NONE, headwise = d.q_mode == ROSAQ_Q_HEADWISE;
  const bool keep_q = rotate && !d.rotation_absorbed;
  const size_t rec_dwords = (c.bits == 4 ? 256 : 192) + 16;
  const size_t wS_bytes = ntiles * ks_s * 64 * 16, wq_bytes = ntiles * G * rec_dwords * 4;
  const size_t qf_bytes = !keep_q ? 0 : (headwise ? (D / kHeadDim) * 8 * 4 * 64 * 16
                                                  : (D / kTileN) * (D / kKStep) * 64 * 16);
  const size_t q_bytes = !rotate ? 0 : (headwise ? D * kHeadDim : D * D) * sizeof(float);

  // the handle's device buffer: [wS | wq | qf | perm | pos]
  struct Part { size_t bytes; void** dst; };
  void *d_perm = nullptr, *d_pos = nullptr;
  Part parts[] = {{wS_bytes, &p->d_wS}, {wq_bytes, &p->d_wq}, {qf_bytes, &p->d_qf},
                  {D * 4, &d_perm}, {D * 4, &d_pos}};
  size_t total = 0;
  for (const Part& q : parts) total += align_up(std::max<size_t>(q.bytes, 16), 256);
  ROSAQ_HIP(hipGetDevice(&p->device));
  ROSAQ_HIP(hipMalloc(&p->d_blob, total));       // owned by the handle from here on (rosaq_free)
  p->blob_bytes = total;
  p->host_only = false;
  size_t off = 0;
  for (const Part& q : parts) {
    *q.dst = static_cast<char*>(p->d_blob) + off;
    off += align_up(std::max<size_t>(q.bytes, 16), 256);
  }
  p->d_perm = static_cast<int32_t*>(d_perm);
  p->d_pos = static_cast<int32_t*>(d_pos);

  // host arrays the canonical form comes back into (sized before the scratch exists: an allocation
  // failure here must not leave it behind)
  c.W_S.resize(N * K); c.codes.resize(N * C); c.scales.resize(N * G); c.zeros.resize(N * G);
  // scratch of this call: [W | What | Q | W_S | codes | scales | zeros | flag]
  const size_t sizes[] = {N * D * 2, rotate ? N * D * 2 : 0, q_bytes, N * K * 2, N * C, N * G * 2, N * G * 2, 256};
  size_t offs[8], tmp_total = 0;
  for (int i = 0; i < 8; ++i) { offs[i] = tmp_total; tmp_total += align_up(std::max<size_t>(sizes[i], 16), 256); }
  char* tmp = nullptr;
  ROSAQ_HIP(hipMalloc(reinterpret_cast<void**>(&tmp), tmp_total));
  unsigned flag = 0;
  hipError_t e = static_cast<size_t>(d.ldw) == D
                     ? hipMemcpyAsync(tmp + offs[0], d.W, N * D * 2, hipMemcpyHostToDevice, st)
                     : hipMemcpy2DAsync(tmp + offs[0], D * 2, d.W, static_cast<size_t>(d.ldw) * 2, D * 2, N,
                                        hipMemcpyHostToDevice, st);
  if (e == hipSuccess && rotate) e = hipMemcpyAsync(tmp + offs[2], d.Q, q_bytes, hipMemcpyHostToDevice, st);
  if (e == hipSuccess) e = hipMemcpyAsync(d_perm, c.perm.data(), D * 4, hipMemcpyHostToDevice, st);
  if (e == hipSuccess) e = hipMemcpyAsync(d_pos, c.pos.data(), D * 4, hipMemcpyHostToDevice, st);
  if (e == hipSuccess) e = hipMemsetAsync(tmp + offs[7], 0, 256, st);
  rc = ROSAQ_OK;
  const char* what = tmp + offs[0];
  if (e == hipSuccess && rotate) {
    rc = launch_rotate_weights_f64(tmp + offs[0], tmp + offs[2], tmp + offs[1], static_cast<int>(N),
                                   static_cast<int>(D), headwise ? 1 : 0, st);
    what = tmp + offs[1];
  }
  if (e == hipSuccess && rc == ROSAQ_OK) {
    QuantPackArgs a{};
    a.what16 = what; a.N = c.N; a.D = c.D; a.K = c.K; a.bits = c.bits; a.perm = p->d_perm;
    a.wS_image = p->d_wS; a.wq_image = p->d_wq;
    a.W_S = tmp + offs[3]; a.codes = tmp + offs[4]; a.scales = tmp + offs[5]; a.zeros = tmp + offs[6];
    a.flag = tmp + offs[7];
    rc = launch_quantize_pack(a, st);
  }
  if (e == hipSuccess && rc == ROSAQ_OK && keep_q)
    rc = launch_rotation_image(tmp + offs[2], c.D, headwise ? 1 : 0, p->d_perm, p->d_qf, st);
  if (e == hipSuccess && rc == ROSAQ_OK) {
    if (N * K) e = hipMemcpyAsync(c.W_S.data(), tmp + offs[3], N * K * 2, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess && N * C) e = hipMemcpyAsync(c.codes.data(), tmp + offs[4], N * C, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess && N * G) e = hipMemcpyAsync(c.scales.data(), tmp + offs[5], N * G * 2, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess && N * G) e = hipMemcpyAsync(c.zeros.data(), tmp + offs[6], N * G * 2, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipMemcpyAsync(&flag, tmp + offs[7], 4, hipMemcpyDeviceToHost, st);
  }
  const hipError_t es = hipStreamSynchronize(st);   // also before the scratch is freed
  if (e == hipSuccess) e = es;
  (void)hipFree(tmp);
  if (rc != ROSAQ_OK) return rc;
  if (e != hipSuccess) {
    set_error(std::string("offline step on the device: ") + hipGetErrorString(e));
    return ROSAQ_ERR_HIP;
  }
  if (flag) return fail(ROSAQ_ERR_NONFINITE, "rotated weight overflows fp16");
  return ROSAQ_OK;
}

static int check_call(const rosaq_packed_t* p, const void* x, int32_t M, int64_t ldx, void* y,
                      int64_t ldy, void* ws, size_t ws_bytes, bool headwise, WsPlan* plan) {
  if (!p) return fail(ROSAQ_ERR_NULL, "handle is NULL");
  if (!x || !y) return fail(ROSAQ_ERR_NULL, "x or y is NULL");
  if ((p->c.q_mode == ROSAQ_Q_HEADWISE) != headwise)
    return fail(ROSAQ_ERR_MODE, headwise ? "rosaq_linear_headwise needs a HEADWISE handle"
                                         : "rosaq_linear does not serve a HEADWISE handle");
  if (M < 1) return fail(ROSAQ_ERR_SHAPE, "M must be at least 1");
  if (M > (1 << 20)) return fail(ROSAQ_ERR_SHAPE, "M above 2^20: split the call");
  // the prologue kernels index the fragment copy of x with 32-bit integers (16 bytes per index)
  if ((static_cast<int64_t>(M) + kMBlock - 1) / kMBlock * kMBlock * p->c.D / 8 > INT32_MAX)
    return fail(ROSAQ_ERR_SHAPE, "M x in_features above 2^34: split the call");
  if (ldx < p->c.D || ldy < p->c.N) return fail(ROSAQ_ERR_SHAPE, "leading dimension smaller than width");
  if (reinterpret_cast<uintptr_t>(x) % 16 || ldx % 8)
    return fail(ROSAQ_ERR_ALIGN, "x must be 16-byte aligned and ldx a multiple of 8");
  if (reinterpret_cast<uintptr_t>(y) % 2) return fail(ROSAQ_ERR_ALIGN, "y must be 2-byte aligned");
  *plan = plan_workspace(*p, M);
  if (!ws || ws_bytes < plan->required) return fail(ROSAQ_ERR_WORKSPACE, "workspace missing or too small");
  if (reinterpret_cast<uintptr_t>(ws) % 256) return fail(ROSAQ_ERR_ALIGN, "workspace must be 256-byte aligned");
  return ROSAQ_OK;
}

static int check_device(const rosaq_packed_t* const* ps, int count) {
  for (int i = 0; i < count; ++i)
    if (ps[i]->host_only) return fail(ROSAQ_ERR_HOSTONLY, "handle was packed with host_only");
  return ROSAQ_OK;
}

// Buffers of one main-GEMM launch.  `chain_*`: a gated pair that feeds a following layer writes its
// product as that layer's input fragments (rosaq_mlp_swiglu) and clears that layer's tickets.
struct GemmIO {
  const void* xf;            // xhat fragments the launch reads
  void* tickets;             // kTicketsPerLaunch words, zero before the launch
  void* part;                // room for partial tiles of a split launch
  size_t part_bytes;
  const int32_t* chain_pos = nullptr;   // device: channel -> storage position of the next layer
  int chain_ks = 0;                     // k-steps of the next layer's input
  void* zero_ptr = nullptr;
  int zero_count = 0;
};

static GemmIO plan_io(const rosaq_packed& p0, const WsPlan& w, char* ws, size_t ws_bytes) {
  GemmIO io{};
  io.xf = ws + (p0.c.q_mode == ROSAQ_Q_FULL ? w.xf_b : w.xf_a);
  io.tickets = ws + w.tickets + kTicketsPerLaunch * sizeof(uint32_t);
  io.part = ws + w.part;
  io.part_bytes = ws_bytes > w.part ? ws_bytes - w.part : 0;
  return io;
}

// y_i = xhat W_i^T for `count` layers that share the xhat fragments `io.xf`.
static int run_main_gemm(const rosaq_packed_t* const* ps, int count, const GemmIO& io, int M,
                         void* const* ys, const int64_t* ldys, void* stream, bool swiglu = false) {
  const Canonical& c = ps[0]->c;
  GemmArgs a{};
  a.xf = io.xf;
  a.nseg = count;
  for (int i = 0; i < count; ++i) {
    const rosaq_packed_t* p = ps[i];
    a.seg[i].wS = p->d_wS; a.seg[i].wq = p->d_wq;
    a.seg[i].out = ys[i]; a.seg[i].ldo = ldys[i]; a.seg[i].N = p->c.N;
  }
  a.M = M;
  a.ks_s = c.K / kKStep; a.G = c.G; a.KS = c.D / kKStep; a.KS_out = 0;
  a.bits = c.bits; a.out_frag = 0;
  if (io.chain_pos) { a.out_frag = 2; a.out_pos = io.chain_pos; a.KS_out = io.chain_ks; }
  a.part = io.part; a.part_bytes = io.part_bytes;
  a.tickets = io.tickets; a.ticket_count = kTicketsPerLaunch;
  a.zero_ptr = io.zero_ptr; a.zero_count = io.zero_count;
  a.swiglu = swiglu ? 1 : 0;
  return launch_gemm(a, g_tune, stream);
}

// x -> xhat fragments in the workspace (gather / head-wise blocks / dense rotation).
static int run_prologue(const rosaq_packed_t* p, const WsPlan& w, const void* x_dev, int M,
                        int64_t ldx, char* ws, size_t ws_bytes, void* hip_stream) {
  const Canonical& c = p->c;
  // the first launch of a call clears the tickets of the GEMM launches behind it
  void* tickets = ws + w.tickets;
  const int n_tickets = 2 * kTicketsPerLaunch;
  if (c.q_mode == ROSAQ_Q_HEADWISE)
    return launch_rotate_headwise(x_dev, ldx, M, c.D, p->d_qf, p->d_pos, ws + w.xf_a, tickets, n_tickets,
                                  hip_stream);
  if (c.q_mode == ROSAQ_Q_NONE)
    return launch_gather(x_dev, ldx, M, c.D, p->d_perm, ws + w.xf_a, tickets, n_tickets, hip_stream);
  // xhat = x fp16(Q), a dense fp16 contraction.
  // rosaq_tune("rot_splits", n >= 2), 17 to 64 rows: slabs of the contraction and a summing launch,
  // when the caller's workspace has room for the partial tiles.  Not the default: measured at
  // 4096^2 and 64 rows, a stream of single calls gains 6 % (17.3 against 18.5 us) but a whole decode
  // step, where other launches sit between the rotations, loses 0.2 % (3.125 against 3.118 ms).
  if (M > 16 && M <= kMBlock && g_tune_rot.splits >= 2) {
    const int slabs = pick_rotate_slabs(c.D, g_tune_rot.splits);
    if (slabs >= 1 && ws_bytes >= w.part + rotate_slab_part_bytes(c.D, slabs))
      return launch_rotate_slabs(x_dev, ldx, M, c.D, p->d_qf, slabs, ws + w.part, ws + w.xf_b, tickets,
                                 n_tickets, hip_stream);
  }
  // the default: one launch of the all-fp16 GEMM whose "weight" is Q^T with rows already in
  // storage order
  GemmArgs a{};
  a.xf = ws + w.xf_a;
  if (M <= 16) {
    a.xrow = x_dev;        // skinny input: the rotation reads x in place, no fragment copy
    a.ldx = ldx;
    // no launch in front of the rotation: it runs unsplit and clears the main GEMM's tickets itself
    a.zero_ptr = static_cast<char*>(tickets) + kTicketsPerLaunch * sizeof(uint32_t);
    a.zero_count = kTicketsPerLaunch;
  } else {
    const int rc = launch_gather(x_dev, ldx, M, c.D, nullptr, ws + w.xf_a, tickets, n_tickets, hip_stream);
    if (rc != ROSAQ_OK) return rc;
  }
  a.nseg = 1;
  a.seg[0].wS = p->d_qf; a.seg[0].wq = nullptr;
  a.seg[0].out = ws + w.xf_b; a.seg[0].ldo = 0; a.seg[0].N = c.D;
  a.M = M;
  a.ks_s = c.D / kKStep; a.G = 0; a.KS = c.D / kKStep; a.KS_out = c.D / kKStep;
  a.bits = 4; a.out_frag = 1;
  GemmTune tune = g_tune_rot;
  tune.splits = 1;           // "rot_splits" selects the slab launches above, never a ticketed split
  return launch_gemm(a, tune, hip_stream);
}

static int run_call(const rosaq_packed_t* const* ps, int count, const void* x_dev, int M,
                    int64_t ldx, void* const* ys, const int64_t* ldys, char* ws, size_t ws_bytes,
                    const WsPlan& w, void* hip_stream, bool swiglu = false) {
  if (g_tune_stages & 1) {
    const int rc = run_prologue(ps[0], w, x_dev, M, ldx, ws, ws_bytes, hip_stream);
    if (rc != ROSAQ_OK) return rc;
  }
  if (!(g_tune_stages & 2)) return ROSAQ_OK;
  return run_main_gemm(ps, count, plan_io(*ps[0], w, ws, ws_bytes), M, ys, ldys, hip_stream, swiglu);
}

static uint64_t fnv1a(uint64_t h, const void* data, size_t n) {
  const unsigned char* b = static_cast<const unsigned char*>(data);
  for (size_t i = 0; i < n; ++i) { h ^= b[i]; h *= 1099511628211ull; }
  return h;
}

}  // namespace rosaq

using namespace rosaq;

extern "C" {

int rosaq_pack_weights(const rosaq_pack_desc* desc, void* hip_stream, rosaq_packed_t** out) {
  if (!out) return fail(ROSAQ_ERR_NULL, "out is NULL");
  *out = nullptr;
  int rc = check_desc(desc);
  if (rc != ROSAQ_OK) return rc;
  rosaq_packed* p = new (std::nothrow) rosaq_packed();
  if (!p) return fail(ROSAQ_ERR_NOMEM, "out of host memory");
  std::string err;
  try {
    if (desc->host_only) {
      rc = pack_host(*desc, &p->c, &err);
      if (rc != ROSAQ_OK) set_error(err);
    } else {
      rc = pack_device(*desc, static_cast<hipStream_t>(hip_stream), p);
    }
  } catch (const std::exception&) { rc = fail(ROSAQ_ERR_NOMEM, "out of host memory"); }
  if (rc != ROSAQ_OK) { rosaq_free(p); return rc; }
  {
    uint64_t h = fnv1a(1469598103934665603ull, &desc->q_mode, sizeof(desc->q_mode));
    h = fnv1a(h, p->c.perm.data(), p->c.perm.size() * sizeof(int32_t));
    if (desc->q_mode == ROSAQ_Q_FULL)
      h = fnv1a(h, desc->Q, sizeof(float) * desc->in_features * static_cast<size_t>(desc->in_features));
    else if (desc->q_mode == ROSAQ_Q_HEADWISE)
      h = fnv1a(h, desc->Q, sizeof(float) * desc->in_features * static_cast<size_t>(kHeadDim));
    p->rot_fingerprint = h;
  }
  if (desc->rotation_absorbed) p->c.q_mode = ROSAQ_Q_NONE;   // run time sees rotated activations
  *out = p;
  return ROSAQ_OK;
}

int rosaq_packed_clone(const rosaq_packed_t* src, void* hip_stream, rosaq_packed_t** out) {
  if (!out) return fail(ROSAQ_ERR_NULL, "out is NULL");
  *out = nullptr;
  if (!src) return fail(ROSAQ_ERR_NULL, "handle is NULL");
  rosaq_packed* p = nullptr;
  try {
    p = new rosaq_packed(*src);
  } catch (const std::bad_alloc&) { return fail(ROSAQ_ERR_NOMEM, "out of host memory"); }
  p->d_blob = nullptr;
  if (!src->host_only) {
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipMalloc(&p->d_blob, src->blob_bytes);
    if (e == hipSuccess)
      e = hipMemcpyAsync(p->d_blob, src->d_blob, src->blob_bytes, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
      set_error(std::string("rosaq_packed_clone: ") + hipGetErrorString(e));
      if (p->d_blob) (void)hipFree(p->d_blob);
      delete p;
      return ROSAQ_ERR_HIP;
    }
    const ptrdiff_t shift = static_cast<char*>(p->d_blob) - static_cast<char*>(src->d_blob);
    auto move = [shift](auto*& q) { q = reinterpret_cast<std::remove_reference_t<decltype(q)>>(
                                        reinterpret_cast<char*>(q) + shift); };
    move(p->d_wS); move(p->d_wq); move(p->d_qf); move(p->d_perm); move(p->d_pos);
  }
  *out = p;
  return ROSAQ_OK;
}

size_t rosaq_workspace_bytes(const rosaq_packed_t* p, int32_t M) {
  if (!p || M < 1) return 0;
  return std::max<size_t>(plan_workspace(*p, M).total, 256);
}

size_t rosaq_workspace_bytes_min(const rosaq_packed_t* p, int32_t M) {
  if (!p || M < 1) return 0;
  return std::max<size_t>(plan_workspace(*p, M).required, 256);
}

size_t rosaq_workspace_bytes_batch(const rosaq_packed_t* const* layers, int32_t count, int32_t M) {
  if (!layers || count < 1 || count > kMaxBatch || M < 1) return 0;
  size_t channels = 0;
  for (int i = 0; i < count; ++i) {
    if (!layers[i]) return 0;
    channels += align_up(static_cast<size_t>(layers[i]->c.N), kTileN);
  }
  return std::max<size_t>(plan_workspace(*layers[0], M, channels).total, 256);
}

int rosaq_linear(const rosaq_packed_t* p, const void* x_dev, int32_t M, int64_t ldx, void* y_dev,
                 int64_t ldy, void* ws_dev, size_t ws_bytes, void* hip_stream) {
  WsPlan w;
  int rc = check_call(p, x_dev, M, ldx, y_dev, ldy, ws_dev, ws_bytes, false, &w);
  if (rc == ROSAQ_OK) rc = check_device(&p, 1);
  if (rc != ROSAQ_OK) return rc;
  return run_call(&p, 1, x_dev, M, ldx, &y_dev, &ldy, static_cast<char*>(ws_dev), ws_bytes, w, hip_stream);
}

int rosaq_linear_headwise(const rosaq_packed_t* p, const void* x_dev, int32_t M, int64_t ldx,
                          void* y_dev, int64_t ldy, void* ws_dev, size_t ws_bytes,
                          void* hip_stream) {
  WsPlan w;
  int rc = check_call(p, x_dev, M, ldx, y_dev, ldy, ws_dev, ws_bytes, true, &w);
  if (rc == ROSAQ_OK) rc = check_device(&p, 1);
  if (rc != ROSAQ_OK) return rc;
  return run_call(&p, 1, x_dev, M, ldx, &y_dev, &ldy, static_cast<char*>(ws_dev), ws_bytes, w, hip_stream);
}

int rosaq_linear_headwise_static(const rosaq_packed_t* p, const void* x_dev, int32_t M, int64_t ldx,
                                 void* y_dev, int64_t ldy, void* hip_stream) {
  if (!p) return fail(ROSAQ_ERR_NULL, "handle is NULL");
  if (M < 1) return fail(ROSAQ_ERR_SHAPE, "M must be at least 1");
  // the size test comes first: it needs no GPU
  const WsPlan need = plan_workspace(*p, M);
  if (need.required > kStaticScratchBytes)
    return fail(ROSAQ_ERR_WORKSPACE, "call needs more scratch than the library's static 8 MiB: use "
                                     "rosaq_linear_headwise with a workspace");
  // the address is only compared against NULL and alignment until the handle has passed its checks
  WsPlan w;
  void* probe = reinterpret_cast<void*>(uintptr_t{256});
  int rc = check_call(p, x_dev, M, ldx, y_dev, ldy, probe, kStaticScratchBytes, true, &w);
  if (rc == ROSAQ_OK) rc = check_device(&p, 1);
  if (rc != ROSAQ_OK) return rc;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != ROSAQ_OK) return rc;
  const size_t ws_bytes = std::min(w.total, kStaticScratchBytes);
  return run_call(&p, 1, x_dev, M, ldx, &y_dev, &ldy, static_cast<char*>(ws), ws_bytes, w, hip_stream);
}

int rosaq_linear_batch(const rosaq_packed_t* const* layers, int32_t count, const void* x_dev,
                       int32_t M, int64_t ldx, void* const* y_dev, const int64_t* ldy,
                       void* ws_dev, size_t ws_bytes, void* hip_stream) {
  if (!layers || !y_dev || !ldy) return fail(ROSAQ_ERR_NULL, "layers, y_dev or ldy is NULL");
  if (count < 1 || count > kMaxBatch) return fail(ROSAQ_ERR_ARG, "count must be between 1 and 4");
  for (int i = 0; i < count; ++i)
    if (!layers[i]) return fail(ROSAQ_ERR_NULL, "a layer handle is NULL");
  const rosaq_packed_t* p0 = layers[0];
  for (int i = 1; i < count; ++i) {
    const Canonical& a = layers[i]->c;
    if (a.D != p0->c.D || a.K != p0->c.K || a.bits != p0->c.bits || a.q_mode != p0->c.q_mode ||
        layers[i]->rot_fingerprint != p0->rot_fingerprint)
      return fail(ROSAQ_ERR_MODE, "layers of a batch must share D, K, bits and the rotation");
  }
  WsPlan w;
  for (int i = 0; i < count; ++i) {
    const int rc = check_call(layers[i], x_dev, M, ldx, y_dev[i], ldy[i], ws_dev, ws_bytes,
                              p0->c.q_mode == ROSAQ_Q_HEADWISE, &w);
    if (rc != ROSAQ_OK) return rc;
  }
  if (check_device(layers, count) != ROSAQ_OK) return ROSAQ_ERR_HOSTONLY;
  return run_call(layers, count, x_dev, M, ldx, y_dev, ldy, static_cast<char*>(ws_dev), ws_bytes, w, hip_stream);
}

int rosaq_linear_swiglu(const rosaq_packed_t* gate, const rosaq_packed_t* up, const void* x_dev, int32_t M,
                        int64_t ldx, void* y_dev, int64_t ldy, void* ws_dev, size_t ws_bytes,
                        void* hip_stream) {
  if (!gate || !up) return fail(ROSAQ_ERR_NULL, "a layer handle is NULL");
  const Canonical &a = gate->c, &b = up->c;
  if (a.N != b.N || a.D != b.D || a.K != b.K || a.bits != b.bits || a.q_mode != b.q_mode ||
      gate->rot_fingerprint != up->rot_fingerprint)
    return fail(ROSAQ_ERR_MODE, "gate and up must share N, D, K, bits and the rotation");
  WsPlan w;
  const bool headwise = a.q_mode == ROSAQ_Q_HEADWISE;
  int rc = check_call(gate, x_dev, M, ldx, y_dev, ldy, ws_dev, ws_bytes, headwise, &w);
  if (rc != ROSAQ_OK) return rc;
  const rosaq_packed_t* ps[2] = {gate, up};
  if (check_device(ps, 2) != ROSAQ_OK) return ROSAQ_ERR_HOSTONLY;
  void* ys[2] = {y_dev, y_dev};
  const int64_t ldys[2] = {ldy, ldy};
  return run_call(ps, 2, x_dev, M, ldx, ys, ldys, static_cast<char*>(ws_dev), ws_bytes, w, hip_stream, true);
}

// Workspace of rosaq_mlp_swiglu: [gate / up: what rosaq_linear_swiglu needs without room for partial
// tiles | down: xhat fragments, tickets | room for the down launch's partial tiles].
struct MlpPlan {
  WsPlan gate;
  size_t down_xf = 0, down_tickets = 0, required = 0, part = 0, total = 0;
};
static MlpPlan plan_mlp(const rosaq_packed& gate, const rosaq_packed& down, int M) {
  MlpPlan m;
  m.gate = plan_workspace(gate, M);
  const size_t mblocks = (static_cast<size_t>(M) + kMBlock - 1) / kMBlock;
  size_t off = m.gate.required;
  m.down_xf = off; off += align_up(mblocks * (down.c.D / kKStep) * 4 * 64 * 16, 256);
  m.down_tickets = off; off += kTicketBytes;
  m.required = off;
  m.part = off;
  off += align_up(part_room(M, down.c.N), 256);
  m.total = off;
  return m;
}

static int check_mlp(const rosaq_packed_t* gate, const rosaq_packed_t* up, const rosaq_packed_t* down) {
  if (!gate || !up || !down) return fail(ROSAQ_ERR_NULL, "a layer handle is NULL");
  const Canonical &a = gate->c, &b = up->c, &d = down->c;
  if (a.N != b.N || a.D != b.D || a.K != b.K || a.bits != b.bits || a.q_mode != b.q_mode ||
      gate->rot_fingerprint != up->rot_fingerprint)
    return fail(ROSAQ_ERR_MODE, "gate and up must share N, D, K, bits and the rotation");
  if (d.D != a.N) return fail(ROSAQ_ERR_SHAPE, "down must take gate's output channels as its input");
  if (d.q_mode != ROSAQ_Q_NONE)
    return fail(ROSAQ_ERR_MODE, "down must run without a run-time rotation (q_mode NONE or rotation_absorbed)");
  return ROSAQ_OK;
}

size_t rosaq_workspace_bytes_mlp(const rosaq_packed_t* gate, const rosaq_packed_t* up,
                                 const rosaq_packed_t* down, int32_t M) {
  if (check_mlp(gate, up, down) != ROSAQ_OK || M < 1) return 0;
  return plan_mlp(*gate, *down, M).total;
}

int rosaq_mlp_swiglu(const rosaq_packed_t* gate, const rosaq_packed_t* up, const rosaq_packed_t* down,
                     const void* x_dev, int32_t M, int64_t ldx, void* y_dev, int64_t ldy, void* ws_dev,
                     size_t ws_bytes, void* hip_stream) {
  int rc = check_mlp(gate, up, down);
  if (rc != ROSAQ_OK) return rc;
  // x against gate, y against down; the workspace is checked against this call's own plan below
  WsPlan unused;
  const bool headwise = gate->c.q_mode == ROSAQ_Q_HEADWISE;
  char* ws = static_cast<char*>(ws_dev);
  rc = check_call(gate, x_dev, M, ldx, y_dev, gate->c.N, ws_dev, ws_bytes, headwise, &unused);
  if (rc != ROSAQ_OK) return rc;
  if (!y_dev) return fail(ROSAQ_ERR_NULL, "y is NULL");
  if (ldy < down->c.N) return fail(ROSAQ_ERR_SHAPE, "leading dimension smaller than width");
  if ((static_cast<int64_t>(M) + kMBlock - 1) / kMBlock * kMBlock * down->c.D / 8 > INT32_MAX)
    return fail(ROSAQ_ERR_SHAPE, "M x in_features above 2^34: split the call");
  const MlpPlan m = plan_mlp(*gate, *down, M);
  if (ws_bytes < m.required) return fail(ROSAQ_ERR_WORKSPACE, "workspace missing or too small");
  const rosaq_packed_t* gu[2] = {gate, up};
  const rosaq_packed_t* all[3] = {gate, up, down};
  if (check_device(all, 3) != ROSAQ_OK) return ROSAQ_ERR_HOSTONLY;
  // 1. xhat of the input (clears the gate / up launch's tickets)
  if (g_tune_stages & 1) {
    rc = run_prologue(gate, m.gate, x_dev, M, ldx, ws, m.gate.required, hip_stream);
    if (rc != ROSAQ_OK) return rc;
  }
  if (!(g_tune_stages & 2)) return ROSAQ_OK;
  // 2. silu(gate) * up, written as down's input fragments at down's storage positions
  GemmIO io = plan_io(*gate, m.gate, ws, m.gate.required);
  io.part = nullptr; io.part_bytes = 0;
  io.chain_pos = down->d_pos; io.chain_ks = down->c.D / kKStep;
  io.zero_ptr = ws + m.down_tickets; io.zero_count = 2 * kTicketsPerLaunch;
  void* hs[2] = {ws + m.down_xf, ws + m.down_xf};
  const int64_t ldh[2] = {0, 0};
  rc = run_main_gemm(gu, 2, io, M, hs, ldh, hip_stream, true);
  if (rc != ROSAQ_OK) return rc;
  // 3. y = h What_down^T
  GemmIO dn{};
  dn.xf = ws + m.down_xf;
  dn.tickets = ws + m.down_tickets + kTicketsPerLaunch * sizeof(uint32_t);
  dn.part = ws + m.part;
  dn.part_bytes = ws_bytes > m.part ? ws_bytes - m.part : 0;
  const int64_t ldys[1] = {ldy};
  return run_main_gemm(&down, 1, dn, M, &y_dev, ldys, hip_stream);
}

int rosaq_packed_info(const rosaq_packed_t* p, int32_t* N, int32_t* D, int32_t* K, int32_t* bits,
                      int32_t* group, int32_t* q_mode, size_t* device_bytes) {
  if (!p) return fail(ROSAQ_ERR_NULL, "handle is NULL");
  if (N) *N = p->c.N;
  if (D) *D = p->c.D;
  if (K) *K = p->c.K;
  if (bits) *bits = p->c.bits;
  if (group) *group = kGroup;
  if (q_mode) *q_mode = p->c.q_mode;
  if (device_bytes) *device_bytes = p->blob_bytes;
  return ROSAQ_OK;
}

int rosaq_packed_export(const rosaq_packed_t* p, int32_t* salient_idx, uint16_t* W_S, uint8_t* codes,
                        uint16_t* scales, uint16_t* zeros) {
  if (!p) return fail(ROSAQ_ERR_NULL, "handle is NULL");
  const Canonical& c = p->c;
  if (salient_idx) std::memcpy(salient_idx, c.salient_idx.data(), c.salient_idx.size() * 4);
  if (W_S) std::memcpy(W_S, c.W_S.data(), c.W_S.size() * 2);
  if (codes) std::memcpy(codes, c.codes.data(), c.codes.size());
  if (scales) std::memcpy(scales, c.scales.data(), c.scales.size() * 2);
  if (zeros) std::memcpy(zeros, c.zeros.data(), c.zeros.size() * 2);
  return ROSAQ_OK;
}

int rosaq_pca_headwise(const void* X_dev, int32_t n_cal, int32_t D, int64_t ldx, float* Q_host,
                       double* eigenvalues_host, void* hip_stream) {
  if (!X_dev || !Q_host || !eigenvalues_host) return fail(ROSAQ_ERR_NULL, "a pointer is NULL");
  if (n_cal < 1 || D < kHeadDim || D % kHeadDim != 0 || ldx < D)
    return fail(ROSAQ_ERR_SHAPE, "n_cal >= 1, D a positive multiple of 128, ldx >= D");
  if (reinterpret_cast<uintptr_t>(X_dev) % 2) return fail(ROSAQ_ERR_ALIGN, "X must be 2-byte aligned");
  try {   // the solver keeps host-side bookkeeping in vectors
    return pca_headwise_device(X_dev, n_cal, D, ldx, Q_host, eigenvalues_host, hip_stream);
  } catch (const std::exception&) { return fail(ROSAQ_ERR_NOMEM, "out of host memory"); }
}

int rosaq_pca_full(const void* X_dev, int32_t n_cal, int32_t D, int64_t ldx, float* Q_host,
                   double* eigenvalues_host, void* hip_stream) {
  if (!X_dev || !Q_host || !eigenvalues_host) return fail(ROSAQ_ERR_NULL, "a pointer is NULL");
  if (n_cal < 1 || D < kGroup || D % kGroup != 0 || D > 8192 || ldx < D)
    return fail(ROSAQ_ERR_SHAPE, "n_cal >= 1, D a multiple of 128 up to 8192, ldx >= D");
  if (reinterpret_cast<uintptr_t>(X_dev) % 2) return fail(ROSAQ_ERR_ALIGN, "X must be 2-byte aligned");
  try {
    return pca_full_device(X_dev, n_cal, D, ldx, Q_host, eigenvalues_host, hip_stream);
  } catch (const std::exception&) { return fail(ROSAQ_ERR_NOMEM, "out of host memory"); }
}

int rosaq_stream_probe(const void* src_dev, size_t src_bytes, const void* shared_dev,
                       size_t shared_bytes, size_t shared_bytes_per_workgroup, int32_t workgroups,
                       int32_t threads, void* sink_dev, size_t sink_bytes, void* hip_stream) {
  if (!src_dev || !sink_dev) return fail(ROSAQ_ERR_NULL, "src_dev or sink_dev is NULL");
  if (workgroups < 1 || threads < 64 || threads > 1024 || threads % 64)
    return fail(ROSAQ_ERR_ARG, "workgroups >= 1 and threads a multiple of 64 up to 1024");
  const size_t waves = static_cast<size_t>(workgroups) * (threads / 64);
  if (src_bytes == 0 || src_bytes % (waves * 1024))
    return fail(ROSAQ_ERR_SHAPE, "src_bytes must be a positive multiple of 1 KiB per wave");
  const size_t wpw = static_cast<size_t>(threads / 64) * 1024;
  if (shared_bytes_per_workgroup % wpw || shared_bytes % 1024)
    return fail(ROSAQ_ERR_SHAPE, "shared sizes must be multiples of 1 KiB (per wave)");
  if (shared_bytes_per_workgroup && (!shared_dev || shared_bytes < shared_bytes_per_workgroup / (threads / 64)))
    return fail(ROSAQ_ERR_SHAPE, "shared buffer missing or smaller than one wave's share");
  if (sink_bytes < waves * 1024) return fail(ROSAQ_ERR_WORKSPACE, "sink smaller than 16 bytes per thread");
  if (reinterpret_cast<uintptr_t>(src_dev) % 16 || reinterpret_cast<uintptr_t>(shared_dev) % 16 ||
      reinterpret_cast<uintptr_t>(sink_dev) % 16)
    return fail(ROSAQ_ERR_ALIGN, "probe buffers must be 16-byte aligned");
  return launch_stream_probe(src_dev, shared_dev, workgroups, threads,
                             static_cast<int>(src_bytes / (waves * 1024)),
                             static_cast<int>(shared_bytes_per_workgroup / wpw),
                             static_cast<int>(shared_bytes / 1024), sink_dev, hip_stream);
}

int rosaq_tune(const char* key, int32_t value) {
  if (!key) return fail(ROSAQ_ERR_NULL, "key is NULL");
  if (!std::strcmp(key, "wpb")) {
    if (value != 0 && value != 4 && value != 8 && value != 16)
      return fail(ROSAQ_ERR_ARG, "wpb must be 0, 4, 8 or 16");
    g_tune.wpb = value; return ROSAQ_OK;
  }
  if (!std::strncmp(key, "rot_", 4) && std::strcmp(key, "rot_splits")) {
    const char* k = key + 4;
    if (value < 0 || value > 4 || value == 3) {
      if (!((std::strcmp(k, "depth") == 0 || std::strcmp(k, "nt") == 0) && value == 3))
        return fail(ROSAQ_ERR_ARG, "bad rotation tuning value");
    }
    if (!std::strcmp(k, "mt")) { g_tune_rot.mt = value; return ROSAQ_OK; }
    if (!std::strcmp(k, "nt")) { g_tune_rot.nt = value; return ROSAQ_OK; }
    if (!std::strcmp(k, "depth")) { g_tune_rot.depth = value; return ROSAQ_OK; }
    return fail(ROSAQ_ERR_ARG, "unknown tuning key");
  }
  if (!std::strcmp(key, "depth")) {
    if (value < 0 || value > 4) return fail(ROSAQ_ERR_ARG, "depth must be 0 to 4");
    g_tune.depth = value; return ROSAQ_OK;
  }
  if (!std::strcmp(key, "splits") || !std::strcmp(key, "rot_splits")) {
    if (value < 0 || value > kMaxSplits) return fail(ROSAQ_ERR_ARG, "splits must be 0 to 16");
    (key[0] == 'r' ? g_tune_rot : g_tune).splits = value; return ROSAQ_OK;
  }
  if (!std::strcmp(key, "mt") || !std::strcmp(key, "nt")) {
    const bool wide = key[0] == 'n' && (value == 3 || value == 6);
    if (value != 0 && value != 1 && value != 2 && value != 4 && !wide)
      return fail(ROSAQ_ERR_ARG, "tile counts must be 0, 1, 2 or 4 (nt also 3 or 6)");
    (key[0] == 'm' ? g_tune.mt : g_tune.nt) = value; return ROSAQ_OK;
  }
  if (!std::strcmp(key, "stages")) {
    if (value < 1 || value > 3) return fail(ROSAQ_ERR_ARG, "stages must be 1, 2 or 3");
    g_tune_stages = value; return ROSAQ_OK;
  }
  return fail(ROSAQ_ERR_ARG, "unknown tuning key");
}

int rosaq_launch_shape(int32_t M, int32_t channels, int32_t in_features, int32_t bits, int32_t* shape_out) {
  if (!shape_out) return fail(ROSAQ_ERR_NULL, "shape_out is NULL");
  if (M < 1 || channels < 1 || channels % kTileN || in_features < kGroup || in_features % kGroup)
    return fail(ROSAQ_ERR_SHAPE, "M >= 1, channels a positive multiple of 16, in_features a positive multiple of 128");
  if (bits != 3 && bits != 4 && bits != 16) return fail(ROSAQ_ERR_ARG, "bits must be 3, 4 or 16");
  const GemmShape s = pick_gemm_shape(M, channels / kTileN, in_features, bits, g_tune,
                                      part_room(M, channels), kTicketsPerLaunch);
  shape_out[0] = s.mt; shape_out[1] = s.nt; shape_out[2] = s.wpb; shape_out[3] = s.depth;
  shape_out[4] = s.splits;
  return ROSAQ_OK;
}

int rosaq_packed_image(const rosaq_packed_t* p, int32_t which, void* out_host, size_t* bytes) {
  if (!p || !bytes) return fail(ROSAQ_ERR_NULL, "handle or bytes is NULL");
  if (which < 0 || which > 3)
    return fail(ROSAQ_ERR_ARG, "which must be 0 / 1 (fp16 fragments / low-bit records rebuilt on the host) or 2 / 3 "
                               "(the same two read back from the device)");
  if (which >= 2) {
    if (p->host_only) return fail(ROSAQ_ERR_HOSTONLY, "handle was packed with host_only");
    const size_t tiles = (static_cast<size_t>(p->c.N) + 127) / 128 * 8;
    const size_t need = which == 2 ? tiles * (p->c.K / kKStep) * 64 * 16
                                   : tiles * p->c.G * ((p->c.bits == 4 ? 256 : 192) + 16) * 4;
    if (out_host) {
      if (*bytes < need) { *bytes = need; return fail(ROSAQ_ERR_WORKSPACE, "image buffer too small"); }
      if (need) ROSAQ_HIP(hipMemcpy(out_host, which == 2 ? p->d_wS : p->d_wq, need, hipMemcpyDeviceToHost));
    }
    *bytes = need;
    return ROSAQ_OK;
  }
  DeviceImage img;
  try {
    build_device_image(p->c, nullptr, &img);
  } catch (const std::exception&) { return fail(ROSAQ_ERR_NOMEM, "out of host memory"); }
  const std::vector<uint32_t>& v = which == 0 ? img.wS : img.wq;
  const size_t need = v.size() * sizeof(uint32_t);
  if (out_host) {
    if (*bytes < need) { *bytes = need; return fail(ROSAQ_ERR_WORKSPACE, "image buffer too small"); }
    if (need) std::memcpy(out_host, v.data(), need);
  }
  *bytes = need;
  return ROSAQ_OK;
}

int rosaq_block_map(int32_t workgroup, int32_t chunks, int32_t row_groups, int32_t* chunk_out, int32_t* row_group_out) {
  if (chunks < 1 || row_groups < 1) return fail(ROSAQ_ERR_SHAPE, "chunks and row_groups must be positive");
  if (workgroup >= 0 && (!chunk_out || !row_group_out)) return fail(ROSAQ_ERR_NULL, "output pointer is NULL");
  int c = -1, m = -1;
  const int r = block_map_host(workgroup, chunks, row_groups, &c, &m);
  if (workgroup < 0) return r;
  *chunk_out = r ? c : -1;
  *row_group_out = r ? m : -1;
  return r;
}

void rosaq_free(rosaq_packed_t* p) {
  if (!p) return;
  if (p->d_blob) (void)hipFree(p->d_blob);
  delete p;
}

const char* rosaq_last_error(void) { return g_error.c_str(); }

}  // extern "C"
