// Offline step of the method on the host (Sec. 3.1-3.3, Eq. 1-3): rotate the
// weight, pick the salient channels, quantise the rest group by group, and lay
// the result out in the order the gfx950 kernels read it.  Pure C++, no GPU calls.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <functional>
#include <exception>
#include <mutex>
#include <numeric>
#include <system_error>
#include <thread>

#include "rosaq_internal.h"

namespace rosaq {

// ---- fp16 conversion -----------------------------------------------------------
double f16_to_f64(uint16_t h) {
  const int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
  double v;
  if (e == 0) v = std::ldexp(static_cast<double>(m), -24);
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = std::ldexp(static_cast<double>(m + 1024), e - 25);
  return sign ? -v : v;
}

// One correctly rounded (half-to-even) step from fp64: scale so that the fp16 ulp
// becomes 1 (a power-of-two scaling, exact), round to integer, reassemble.
uint16_t f64_to_f16(double v) {
  const uint16_t sign = std::signbit(v) ? 0x8000u : 0u;
  if (std::isnan(v)) return sign | 0x7e00u;
  const double a = std::fabs(v);
  if (a >= 65520.0) return sign | 0x7c00u;        // rounds to infinity
  if (a < std::ldexp(1.0, -14)) {                 // subnormal range: ulp 2^-24
    const double m = std::nearbyint(std::ldexp(a, 24));
    return sign | static_cast<uint16_t>(m);       // m == 1024 is the smallest normal
  }
  int e;
  std::frexp(a, &e);                              // a = f * 2^e, f in [0.5, 1)
  e -= 1;                                         // a in [2^e, 2^(e+1))
  double m = std::nearbyint(std::ldexp(a, 10 - e));   // in [1024, 2048]
  if (m >= 2048.0) { m = 1024.0; e += 1; }
  return sign | static_cast<uint16_t>(((e + 15) << 10) + (static_cast<int>(m) - 1024));
}

// ---- What = W Q in fp64 (Eq. 1, [out, in] layout) ------------------------------
namespace {

// out[r][c] += sum_k a[r][k] * b[k][c] for a KB x CB tile of b and RB rows.
__attribute__((target_clones("arch=haswell", "default")))
void tile_kernel(const double* a, int lda, const double* b, int ldb, double* o, int ldo,
                 int rows, int kb, int cb) {
  for (int r = 0; r < rows; ++r) {
    double* orow = o + static_cast<size_t>(r) * ldo;
    const double* arow = a + static_cast<size_t>(r) * lda;
    for (int k = 0; k < kb; ++k) {
      const double w = arow[k];
      const double* brow = b + static_cast<size_t>(k) * ldb;
      for (int c = 0; c < cb; ++c) orow[c] += w * brow[c];
    }
  }
}

// Runs fn over [0, n) in slices on up to 32 threads.  An exception thrown by a slice (an
// allocation that fails) is carried to the calling thread and thrown again there after every
// thread has joined; if a thread cannot be started the remaining rows run on the calling thread.
void parallel_rows(int n, const std::function<void(int, int)>& fn) {
  unsigned hw = std::thread::hardware_concurrency();
  int nt = static_cast<int>(std::min<unsigned>(hw ? hw : 1u, 32u));
  nt = std::max(1, std::min(nt, n / 4 > 0 ? n / 4 : 1));
  if (nt == 1) { fn(0, n); return; }
  std::vector<std::thread> th;
  std::exception_ptr first;
  std::mutex mu;
  auto guarded = [&](int lo, int hi) {
    try {
      fn(lo, hi);
    } catch (...) {
      std::lock_guard<std::mutex> lock(mu);
      if (!first) first = std::current_exception();
    }
  };
  const int chunk = (n + nt - 1) / nt;
  for (int t = 0; t < nt; ++t) {
    const int lo = t * chunk, hi = std::min(n, lo + chunk);
    if (lo >= hi) break;
    try {
      th.emplace_back(guarded, lo, hi);
    } catch (const std::system_error&) {
      guarded(lo, n);   // no more threads: finish here
      break;
    }
  }
  for (auto& t : th) t.join();
  if (first) std::rethrow_exception(first);
}

// Dense rotation: out [N x D] fp64 = W (fp16) * Q (fp32 [D x D] row-major).
void rotate_full(const rosaq_pack_desc& d, std::vector<double>* out) {
  const int N = d.out_features, D = d.in_features;
  out->assign(static_cast<size_t>(N) * D, 0.0);
  constexpr int KB = 128, CB = 512;
  parallel_rows(N, [&](int lo, int hi) {
    std::vector<double> qt(static_cast<size_t>(KB) * CB);
    std::vector<double> wt;
    const int rows = hi - lo;
    wt.resize(static_cast<size_t>(rows) * KB);
    for (int c0 = 0; c0 < D; c0 += CB) {
      const int cb = std::min(CB, D - c0);
      for (int k0 = 0; k0 < D; k0 += KB) {
        const int kb = std::min(KB, D - k0);
        for (int k = 0; k < kb; ++k)
          for (int c = 0; c < cb; ++c)
            qt[static_cast<size_t>(k) * CB + c] =
                static_cast<double>(d.Q[static_cast<size_t>(k0 + k) * D + c0 + c]);
        for (int r = 0; r < rows; ++r)
          for (int k = 0; k < kb; ++k)
            wt[static_cast<size_t>(r) * KB + k] =
                f16_to_f64(d.W[static_cast<size_t>(lo + r) * d.ldw + k0 + k]);
        tile_kernel(wt.data(), KB, qt.data(), CB, out->data() + static_cast<size_t>(lo) * D + c0,
                    D, rows, kb, cb);
      }
    }
  });
}

// Block-diagonal rotation (Eq. 6): out[:, 128h..] = W[:, 128h..] * Q_h.
void rotate_headwise(const rosaq_pack_desc& d, std::vector<double>* out) {
  const int N = d.out_features, D = d.in_features, H = D / kHeadDim;
  out->assign(static_cast<size_t>(N) * D, 0.0);
  parallel_rows(N, [&](int lo, int hi) {
    std::vector<double> qh(kHeadDim * kHeadDim), wt(kHeadDim);
    for (int h = 0; h < H; ++h) {
      const float* q = d.Q + static_cast<size_t>(h) * kHeadDim * kHeadDim;
      for (int i = 0; i < kHeadDim * kHeadDim; ++i) qh[i] = static_cast<double>(q[i]);
      for (int n = lo; n < hi; ++n) {
        for (int k = 0; k < kHeadDim; ++k)
          wt[k] = f16_to_f64(d.W[static_cast<size_t>(n) * d.ldw + h * kHeadDim + k]);
        tile_kernel(wt.data(), kHeadDim, qh.data(), kHeadDim,
                    out->data() + static_cast<size_t>(n) * D + h * kHeadDim, D, 1, kHeadDim,
                    kHeadDim);
      }
    }
  });
}

}  // namespace

// Salient channels (Sec. 3.2; per-head and ablation rules of the appendices) and the storage
// order [salient ; rest ascending].  Fills the shape fields, salient_idx, perm and pos.
void pack_select(const rosaq_pack_desc& d, Canonical* c) {
  const int N = d.out_features, D = d.in_features, K = d.K;
  c->N = N; c->D = D; c->K = K; c->bits = d.bits; c->q_mode = d.q_mode;
  c->G = (D - K) / kGroup;
  // Every rule ranks channels by eigenvalue with ties going to the lower channel.
  std::vector<char> is_sal(D, 0);
  {
    const double* lam = d.eigenvalues;
    auto ranked = [&](int lo, int hi, bool largest_first) {
      std::vector<int32_t> idx(hi - lo);
      std::iota(idx.begin(), idx.end(), lo);
      std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) {
        return largest_first ? lam[a] > lam[b] : lam[a] < lam[b];
      });
      return idx;
    };
    switch (d.select_rule) {
      case ROSAQ_SELECT_TOP_PER_HEAD: {
        const int H = D / kHeadDim, per = K / H;
        for (int h = 0; h < H; ++h) {
          const std::vector<int32_t> r = ranked(h * kHeadDim, (h + 1) * kHeadDim, true);
          for (int i = 0; i < per; ++i) is_sal[r[i]] = 1;
        }
        break;
      }
      case ROSAQ_SELECT_BOTTOM: {
        const std::vector<int32_t> r = ranked(0, D, false);
        for (int i = 0; i < K; ++i) is_sal[r[i]] = 1;
        break;
      }
      case ROSAQ_SELECT_CONSECUTIVE:
        for (int i = 0; i < K; ++i) is_sal[d.select_arg + i] = 1;
        break;
      case ROSAQ_SELECT_TOP_AND_BOTTOM: {
        const std::vector<int32_t> top = ranked(0, D, true), bottom = ranked(0, D, false);
        for (int i = 0; i < K / 2; ++i) is_sal[top[i]] = 1;
        int taken = 0;
        for (int i = 0; i < D && taken < K / 2; ++i)
          if (!is_sal[bottom[i]]) { is_sal[bottom[i]] = 2; ++taken; }
        break;
      }
      default: {
        const std::vector<int32_t> r = ranked(0, D, true);
        for (int i = 0; i < K; ++i) is_sal[r[i]] = 1;
      }
    }
  }
  c->salient_idx.clear(); c->perm.clear();
  for (int ch = 0; ch < D; ++ch) if (is_sal[ch]) c->salient_idx.push_back(ch);
  c->perm = c->salient_idx;
  for (int ch = 0; ch < D; ++ch) if (!is_sal[ch]) c->perm.push_back(ch);
  c->pos.assign(D, 0);
  for (int p = 0; p < D; ++p) c->pos[c->perm[p]] = p;
}

// Input checks that need the data: every eigenvalue, weight and rotation entry finite.
int pack_validate(const rosaq_pack_desc& d, std::string* err) {
  const int N = d.out_features, D = d.in_features;
  for (int i = 0; i < D; ++i)
    if (!std::isfinite(d.eigenvalues[i])) { *err = "eigenvalues contain NaN/Inf"; return ROSAQ_ERR_NONFINITE; }
  std::atomic<bool> bad{false};
  parallel_rows(N, [&](int lo, int hi) {
    bool local = false;
    for (int n = lo; n < hi; ++n)
      for (int k = 0; k < D; ++k)
        if (((d.W[static_cast<size_t>(n) * d.ldw + k] >> 10) & 31) == 31) local = true;
    if (local) bad.store(true, std::memory_order_relaxed);
  });
  if (bad.load()) { *err = "W contains NaN/Inf"; return ROSAQ_ERR_NONFINITE; }
  if (d.q_mode != ROSAQ_Q_NONE) {
    const int rows = d.q_mode == ROSAQ_Q_FULL ? D : kHeadDim;    // Q as [D][rows]
    parallel_rows(D, [&](int lo, int hi) {
      bool local = false;
      for (size_t i = static_cast<size_t>(lo) * rows; i < static_cast<size_t>(hi) * rows; ++i)
        if (!std::isfinite(d.Q[i])) local = true;
      if (local) bad.store(true, std::memory_order_relaxed);
    });
    if (bad.load()) { *err = "Q contains NaN/Inf"; return ROSAQ_ERR_NONFINITE; }
  }
  return ROSAQ_OK;
}

int pack_host(const rosaq_pack_desc& d, Canonical* c, std::string* err,
              const std::vector<uint16_t>* rotated16) {
  const int N = d.out_features, D = d.in_features, K = d.K;
  const int rcv = pack_validate(d, err);
  if (rcv != ROSAQ_OK) return rcv;
  c->G = (D - K) / kGroup;

  // 1. rotate, round once to fp16
  std::vector<uint16_t> what_local;
  if (rotated16 == nullptr) what_local.resize(static_cast<size_t>(N) * D);
  std::vector<uint16_t>& what_rw = what_local;
  if (rotated16 != nullptr) {
    for (uint16_t h : *rotated16)
      if (((h >> 10) & 31) == 31) { *err = "rotated weight overflows fp16"; return ROSAQ_ERR_NONFINITE; }
  } else if (d.q_mode == ROSAQ_Q_NONE) {
    for (int n = 0; n < N; ++n)
      std::memcpy(&what_rw[static_cast<size_t>(n) * D], d.W + static_cast<size_t>(n) * d.ldw,
                  sizeof(uint16_t) * D);
  } else {
    std::vector<double> rot;
    try {
      if (d.q_mode == ROSAQ_Q_FULL) rotate_full(d, &rot); else rotate_headwise(d, &rot);
    } catch (const std::bad_alloc&) { *err = "out of host memory"; return ROSAQ_ERR_NOMEM; }
    std::atomic<bool> bad{false};
    parallel_rows(N, [&](int lo, int hi) {
      bool local_bad = false;
      for (size_t i = static_cast<size_t>(lo) * D; i < static_cast<size_t>(hi) * D; ++i) {
        what_rw[i] = f64_to_f16(rot[i]);
        if (((what_rw[i] >> 10) & 31) == 31) local_bad = true;
      }
      if (local_bad) bad.store(true, std::memory_order_relaxed);
    });
    if (bad.load()) { *err = "rotated weight overflows fp16"; return ROSAQ_ERR_NONFINITE; }
  }
  const std::vector<uint16_t>& what = rotated16 ? *rotated16 : what_local;

  // 2. salient channels and storage order
  pack_select(d, c);

  // 3-4. split and quantise (Eq. 3, Sec. 3.3)
  const int G = c->G, C = D - K;
  const double qmax = static_cast<double>((1 << d.bits) - 1);
  c->W_S.assign(static_cast<size_t>(N) * K, 0);
  c->codes.assign(static_cast<size_t>(N) * C, 0);
  c->scales.assign(static_cast<size_t>(N) * G, 0);
  c->zeros.assign(static_cast<size_t>(N) * G, 0);
  parallel_rows(N, [&](int lo, int hi) {
    double w[kGroup];
    for (int n = lo; n < hi; ++n) {
      const uint16_t* row = &what[static_cast<size_t>(n) * D];
      for (int i = 0; i < K; ++i) c->W_S[static_cast<size_t>(n) * K + i] = row[c->perm[i]];
      for (int j = 0; j < G; ++j) {
        double mx = -INFINITY, mn = INFINITY;
        for (int i = 0; i < kGroup; ++i) {
          w[i] = f16_to_f64(row[c->perm[K + j * kGroup + i]]);
          mx = std::max(mx, w[i]); mn = std::min(mn, w[i]);
        }
        const uint16_t s16 = f64_to_f16(std::max((mx - mn) / qmax, std::ldexp(1.0, -14)));
        const double s = f16_to_f64(s16);
        const double z = std::min(std::max(std::nearbyint(-mn / s), 0.0), qmax);
        c->scales[static_cast<size_t>(n) * G + j] = s16;
        c->zeros[static_cast<size_t>(n) * G + j] = f64_to_f16(z);
        uint8_t* q = &c->codes[static_cast<size_t>(n) * C + j * kGroup];
        for (int i = 0; i < kGroup; ++i)
          q[i] = static_cast<uint8_t>(std::min(std::max(std::nearbyint(w[i] / s) + z, 0.0), qmax));
      }
    }
  });
  return ROSAQ_OK;
}

// ---- device layout --------------------------------------------------------------
// One v_mfma_f32_16x16x32_f16 operand fragment: lane l supplies 8 halves for
// (row or column l % 16, contraction indices 8*(l/16) .. 8*(l/16)+7).  Every
// operand array below is a sequence of such 64-lane fragments so that a wave
// reads one fragment with one fully coalesced load per lane.
void build_device_image(const Canonical& c, const float* Q, DeviceImage* img) {
  const int N = c.N, D = c.D, K = c.K, G = c.G;
  const int ntiles = ((N + 127) / 128) * 8;   // whole 128-channel chunks, zero padded
  const int ks_s = K / kKStep;
  const int C = D - K;

  // salient fp16 fragments: [tile][ks][lane][8 halves]
  img->wS.assign(static_cast<size_t>(ntiles) * ks_s * 64 * 4, 0);
  {
    uint16_t* h = reinterpret_cast<uint16_t*>(img->wS.data());
    parallel_rows(ntiles, [&](int t_lo, int t_hi) {
    for (int t = t_lo; t < t_hi; ++t)
      for (int ks = 0; ks < ks_s; ++ks)
        for (int lane = 0; lane < 64; ++lane) {
          const int n = t * kTileN + (lane & 15), j = lane >> 4;
          if (n >= N) continue;
          uint16_t* dst = h + ((static_cast<size_t>(t) * ks_s + ks) * 64 + lane) * 8;
          for (int e = 0; e < 8; ++e)
            dst[e] = c.W_S[static_cast<size_t>(n) * K + ks * kKStep + j * 8 + e];
        }
    });
  }

  // scale | zero << 16 : [tile][g][16]
  img->sz.assign(static_cast<size_t>(ntiles) * G * 16, 0x00000400u /* scale 2^-14, zero 0 */);
  for (int t = 0; t < ntiles; ++t)
    for (int g = 0; g < G; ++g)
      for (int r = 0; r < 16; ++r) {
        const int n = t * kTileN + r;
        if (n >= N) continue;
        img->sz[(static_cast<size_t>(t) * G + g) * 16 + r] =
            static_cast<uint32_t>(c.scales[static_cast<size_t>(n) * G + g]) |
            (static_cast<uint32_t>(c.zeros[static_cast<size_t>(n) * G + g]) << 16);
      }

  // low-bit fragments.  A lane owns, per group, 32 codes: 4 k-steps x 8 elements,
  // element e of k-step t being storage column g*128 + t*32 + 8*(lane/16) + e.
  if (c.bits == 4) {
    // dword t holds k-step t; element e sits in nibble (e >> 1) + 4 * (e & 1), so
    // that (v >> 4i) & 0x000f000f is the fp16 pair (e = 2i, e = 2i + 1).
    img->wq.assign(static_cast<size_t>(ntiles) * G * 64 * 4, 0);
    parallel_rows(ntiles, [&](int t_lo, int t_hi) {
    for (int t = t_lo; t < t_hi; ++t)
      for (int g = 0; g < G; ++g)
        for (int lane = 0; lane < 64; ++lane) {
          const int n = t * kTileN + (lane & 15), j = lane >> 4;
          if (n >= N) continue;
          const uint8_t* q = &c.codes[static_cast<size_t>(n) * C + g * kGroup + j * 8];
          uint32_t* dst = &img->wq[((static_cast<size_t>(t) * G + g) * 64 + lane) * 4];
          for (int ks = 0; ks < 4; ++ks) {
            uint32_t v = 0;
            for (int e = 0; e < 8; ++e)
              v |= static_cast<uint32_t>(q[ks * kKStep + e] & 15) << (4 * ((e >> 1) + 4 * (e & 1)));
            dst[ks] = v;
          }
        }
    });
  } else {
    // INT3, 32 codes of a lane and group in 3 dwords.  The 16 fp16 pairs P = 4 * ks + i
    // (elements 2i and 2i+1 of k-step ks) are laid out for a mask-and-or extraction into an
    // fp16 mantissa: pair P < 15 sits in dword P / 5 at bit 3 * (P % 5) (element 2i) and
    // 16 + 3 * (P % 5) (element 2i+1); pair 15 is spread over the spare bits 15 / 31 of the
    // three dwords, code bit b in dword b.
    img->wq.assign(static_cast<size_t>(ntiles) * G * 64 * 3, 0);
    parallel_rows(ntiles, [&](int t_lo, int t_hi) {
    for (int t = t_lo; t < t_hi; ++t)
      for (int g = 0; g < G; ++g)
        for (int lane = 0; lane < 64; ++lane) {
          const int n = t * kTileN + (lane & 15), j = lane >> 4;
          if (n >= N) continue;
          const uint8_t* q = &c.codes[static_cast<size_t>(n) * C + g * kGroup + j * 8];
          uint32_t* dst = &img->wq[((static_cast<size_t>(t) * G + g) * 64 + lane) * 3];
          uint32_t w[3] = {0, 0, 0};
          for (int ks = 0; ks < 4; ++ks)
            for (int e = 0; e < 8; ++e) {
              const uint32_t code = q[ks * kKStep + e] & 7;
              const int P = 4 * ks + (e >> 1), half = (e & 1) * 16;
              if (P < 15) {
                w[P / 5] |= code << (half + 3 * (P % 5));
              } else {
                for (int b = 0; b < 3; ++b) w[b] |= ((code >> b) & 1u) << (half + 15);
              }
            }
          dst[0] = w[0]; dst[1] = w[1]; dst[2] = w[2];
        }
    });
  }

  // One record per (tile, group): the code fragment followed by the 16 scale|zero words,
  // so a wave finds both in adjacent cache lines (1088 bytes INT4, 832 bytes INT3).
  {
    const size_t cw = c.bits == 4 ? 256 : 192, rw = cw + 16;
    std::vector<uint32_t> rec(static_cast<size_t>(ntiles) * G * rw);
    for (size_t r = 0; r < static_cast<size_t>(ntiles) * G; ++r) {
      std::memcpy(&rec[r * rw], &img->wq[r * cw], cw * 4);
      std::memcpy(&rec[r * rw + cw], &img->sz[r * 16], 16 * 4);
    }
    img->wq.swap(rec);
    std::vector<uint32_t>().swap(img->sz);
  }

  // fp16 rotation fragments (skipped when the caller has no Q at hand and only wants the weights)
  img->qf.clear();
  if (Q == nullptr) return;
  if (c.q_mode == ROSAQ_Q_FULL) {
    // rotation as a linear layer with "weight" Q^T, output columns already in
    // storage order: fragment row p is rotated channel perm[p].
    const int ct = D / kTileN, ks_n = D / kKStep;
    img->qf.assign(static_cast<size_t>(ct) * ks_n * 64 * 4, 0);
    uint16_t* h = reinterpret_cast<uint16_t*>(img->qf.data());
    parallel_rows(ct, [&](int lo, int hi) {
      for (int t = lo; t < hi; ++t)
        for (int ks = 0; ks < ks_n; ++ks)
          for (int lane = 0; lane < 64; ++lane) {
            const int ch = c.perm[t * kTileN + (lane & 15)], j = lane >> 4;
            uint16_t* dst = h + ((static_cast<size_t>(t) * ks_n + ks) * 64 + lane) * 8;
            for (int e = 0; e < 8; ++e)
              dst[e] = f64_to_f16(static_cast<double>(
                  Q[static_cast<size_t>(ks * kKStep + j * 8 + e) * D + ch]));
          }
    });
  } else if (c.q_mode == ROSAQ_Q_HEADWISE) {
    // [head][column tile ct][k-step t][lane]: element e = Q_h[32t + 8(lane/16) + e][16ct + lane%16]
    const int H = D / kHeadDim;
    img->qf.assign(static_cast<size_t>(H) * 8 * 4 * 64 * 4, 0);
    uint16_t* h = reinterpret_cast<uint16_t*>(img->qf.data());
    for (int hd = 0; hd < H; ++hd)
      for (int ct = 0; ct < 8; ++ct)
        for (int t = 0; t < 4; ++t)
          for (int lane = 0; lane < 64; ++lane) {
            const int col = ct * 16 + (lane & 15), j = lane >> 4;
            uint16_t* dst = h + ((((static_cast<size_t>(hd) * 8 + ct) * 4 + t) * 64) + lane) * 8;
            for (int e = 0; e < 8; ++e)
              dst[e] = f64_to_f16(static_cast<double>(
                  Q[(static_cast<size_t>(hd) * kHeadDim + t * kKStep + j * 8 + e) * kHeadDim + col]));
          }
  }
}

}  // namespace rosaq
