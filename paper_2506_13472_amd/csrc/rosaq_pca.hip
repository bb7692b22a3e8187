// Head-wise PCA on the GPU (Sec. 3.1 Eq. 4, Sec. 3.1.1): per 128-channel head the
// uncentred second moment C_h = X_h^T X_h / n_cal in fp64 and its eigen-decomposition by
// cyclic Jacobi rotations, one workgroup per head with the 128 x 128 matrix in LDS.
// Calibration-time code: it allocates its own scratch and waits for the result.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <numeric>
#include <string>
#include <vector>

#include "rosaq_internal.h"

namespace rosaq {

constexpr int kH = 128;        // head dimension
constexpr int kLd = kH + 1;    // padded LDS row stride (doubles): column walks hit distinct banks

// C_h[i][j] = sum_r X[r][h*128+i] * X[r][h*128+j] / n_cal, rows added in increasing r.
// One workgroup per head, thread t owns the 8 x 8 block (t / 16, t % 16).
__global__ __launch_bounds__(256) void second_moment_kernel(const _Float16* __restrict__ X,
                                                            int64_t ldx, int n_cal,
                                                            double* __restrict__ C) {
  __shared__ double row[kH];
  const int h = blockIdx.x;
  const int bi = (threadIdx.x >> 4) * 8, bj = (threadIdx.x & 15) * 8;
  double acc[8][8] = {};
  for (int r = 0; r < n_cal; ++r) {
    __syncthreads();
    if (threadIdx.x < kH)
      row[threadIdx.x] = static_cast<double>(X[static_cast<int64_t>(r) * ldx + h * kH + threadIdx.x]);
    __syncthreads();
    double a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = row[bi + i]; b[i] = row[bj + i]; }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_fma(a[i], b[j], acc[i][j]);
  }
  double* out = C + static_cast<size_t>(h) * kH * kH;
  const double inv = 1.0 / static_cast<double>(n_cal);
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) out[(bi + i) * kH + bj + j] = acc[i][j] * inv;
}

// Cyclic Jacobi on one symmetric 128 x 128 matrix per workgroup.  A round rotates 64
// disjoint (p, q) planes at once (round-robin tournament order, 127 rounds per sweep):
// angles from the current a_pp, a_qq, a_pq; then A <- J^T A J (columns, then rows) and
// V <- V J.  Entries already at round-off level are set to zero instead of rotated.
// Stops when the off-diagonal Frobenius norm is <= tol * ||A||_F or after max_sweeps.
__global__ __launch_bounds__(1024) void jacobi128_kernel(const double* __restrict__ C,
                                                         double* __restrict__ V_out,
                                                         double* __restrict__ lam_out,
                                                         int* __restrict__ sweeps_out, double tol,
                                                         int max_sweeps) {
  extern __shared__ double lds[];
  double* A = lds;                         // [128][129]
  double* cs = lds + kH * kLd;             // [64] cos, [64] sin
  int* pq = reinterpret_cast<int*>(cs + 128);   // [64] p, [64] q
  double* red = reinterpret_cast<double*>(pq + 128);   // [16] reduction scratch
  const int h = blockIdx.x, tid = threadIdx.x;
  double* V = V_out + static_cast<size_t>(h) * kH * kH;   // row-major [i][j], column j = vector j
  const double* Ch = C + static_cast<size_t>(h) * kH * kH;

  for (int i = tid; i < kH * kH; i += 1024) {
    const int r = i >> 7, c = i & 127;
    A[r * kLd + c] = 0.5 * (Ch[r * kH + c] + Ch[c * kH + r]);
    V[i] = r == c ? 1.0 : 0.0;
  }
  __syncthreads();

  auto block_sum = [&](double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    double s = 0.0;
    for (int w = 0; w < 16; ++w) s += red[w];
    return s;
  };
  double part = 0.0;
  for (int i = tid; i < kH * kH; i += 1024) { const double a = A[(i >> 7) * kLd + (i & 127)]; part += a * a; }
  const double norm2 = block_sum(part);
  const double tiny = 2.220446049250313e-16 * sqrt(norm2) / kH;
  int sweep = 0;
  int converged = norm2 > 0.0 ? 0 : 1;
  if (norm2 > 0.0) {
    // the test runs before every sweep and once more after the last one
    for (;; ++sweep) {
      part = 0.0;
      for (int i = tid; i < kH * kH; i += 1024) {
        const int r = i >> 7, c = i & 127;
        if (r != c) { const double a = A[r * kLd + c]; part += a * a; }
      }
      const double off2 = block_sum(part);
      if (off2 <= tol * tol * norm2) { converged = 1; break; }
      if (sweep == max_sweeps) break;
      for (int round = 0; round < kH - 1; ++round) {
        // tournament: player 127 stays, players 0..126 rotate; slot k meets slot 127 - k
        if (tid < 64) {
          auto player = [&](int slot) { return slot == kH - 1 ? kH - 1 : (slot + round) % (kH - 1); };
          const int a = player(tid), b = player(kH - 1 - tid);
          const int p = a < b ? a : b, q = a < b ? b : a;
          const double apq = A[p * kLd + q], app = A[p * kLd + p], aqq = A[q * kLd + q];
          double c = 1.0, s = 0.0;
          if (fabs(apq) > tiny) {
            const double tau = (aqq - app) / (2.0 * apq);
            const double t = tau == 0.0 ? 1.0 : copysign(1.0, tau) / (fabs(tau) + hypot(1.0, tau));
            c = 1.0 / sqrt(1.0 + t * t);
            s = t * c;
          } else {
            A[p * kLd + q] = 0.0;
            A[q * kLd + p] = 0.0;
          }
          cs[tid] = c; cs[64 + tid] = s; pq[tid] = p; pq[64 + tid] = q;
        }
        __syncthreads();
        // columns of A and of V: (x_p, x_q) <- (c x_p - s x_q, s x_p + c x_q) for every row
        for (int w = tid; w < 64 * kH; w += 1024) {
          const int k = w >> 7, i = w & 127;
          const double c = cs[k], s = cs[64 + k];
          const int p = pq[k], q = pq[64 + k];
          const double ap = A[i * kLd + p], aq = A[i * kLd + q];
          A[i * kLd + p] = c * ap - s * aq;
          A[i * kLd + q] = s * ap + c * aq;
          const double vp = V[i * kH + p], vq = V[i * kH + q];
          V[i * kH + p] = c * vp - s * vq;
          V[i * kH + q] = s * vp + c * vq;
        }
        __syncthreads();
        // rows of A
        for (int w = tid; w < 64 * kH; w += 1024) {
          const int k = w >> 7, j = w & 127;
          const double c = cs[k], s = cs[64 + k];
          const int p = pq[k], q = pq[64 + k];
          const double ap = A[p * kLd + j], aq = A[q * kLd + j];
          A[p * kLd + j] = c * ap - s * aq;
          A[q * kLd + j] = s * ap + c * aq;
        }
        __syncthreads();
      }
    }
  }
  if (tid < kH) lam_out[h * kH + tid] = A[tid * kLd + tid];
  if (tid == 0) sweeps_out[h] = converged ? sweep : -1;
}

// ---- layer-wise PCA (Sec. 3.1, Eq. 4) for a whole layer: one-sided Jacobi -----------------------
// The eigenvectors of C = X^T X / n_cal are the right singular vectors of X, its eigenvalues the
// squared column norms of X V / n_cal.  Plane rotations are applied to pairs of columns of X (kept
// transposed, Y[c][:] = column c, so that a column is contiguous) until all columns are mutually
// orthogonal; the same rotations accumulate in V.  C itself (D x D) is never formed and no
// rotation touches more than two rows of Y and V, so the D / 2 disjoint pairs of a round run on
// D / 2 workgroups with no exchange at all -- one launch per round, D - 1 rounds per sweep.

// Y[c][r] = X[r][c] in fp64 (rows padded with zeros to n_pad), Vt = I.
__global__ __launch_bounds__(256) void hestenes_init_kernel(const _Float16* __restrict__ X, int64_t ldx,
                                                            int n_cal, int n_pad, int D,
                                                            double* __restrict__ Y, double* __restrict__ Vt) {
  const int c = blockIdx.x;
  for (int r = threadIdx.x; r < n_pad; r += 256)
    Y[static_cast<size_t>(c) * n_pad + r] = r < n_cal ? static_cast<double>(X[static_cast<int64_t>(r) * ldx + c]) : 0.0;
  for (int j = threadIdx.x; j < D; j += 256) Vt[static_cast<size_t>(c) * D + j] = j == c ? 1.0 : 0.0;
}

// One round: workgroup k rotates the pair (p, q) that the round-robin tournament assigns to it
// (player D - 1 stays, the others move one seat per round; seat k meets seat D - 1 - k).
//   alpha = |y_p|^2, beta = |y_q|^2, gamma = y_p . y_q;  zeta = (beta - alpha) / (2 gamma),
//   t = sign(zeta) / (|zeta| + sqrt(1 + zeta^2)), c = 1 / sqrt(1 + t^2), s = c t,
//   (y_p, y_q) <- (c y_p - s y_q, s y_p + c y_q), the same for the rows p, q of Vt.
// Pairs that are orthogonal to round-off (|gamma| <= eps sqrt(alpha beta)) are left alone.
// gamma^2 of every pair (before its rotation) and, in the first round of a sweep, alpha^2 + beta^2
// go to `stats` slots that a later launch adds up in a fixed order.
__global__ __launch_bounds__(256) void hestenes_round_kernel(double* __restrict__ Y, double* __restrict__ Vt,
                                                             int n_pad, int D, int round,
                                                             double* __restrict__ gamma2,
                                                             double* __restrict__ diag2) {
  __shared__ double red[3][4];
  const int k = blockIdx.x, tid = threadIdx.x;
  auto player = [&](int seat) { return seat == D - 1 ? D - 1 : (seat + round) % (D - 1); };
  const int a = player(k), b = player(D - 1 - k);
  const int p = a < b ? a : b, q = a < b ? b : a;
  double* yp = Y + static_cast<size_t>(p) * n_pad;
  double* yq = Y + static_cast<size_t>(q) * n_pad;
  double al = 0.0, be = 0.0, ga = 0.0;
  for (int r = tid; r < n_pad; r += 256) {
    const double u = yp[r], v = yq[r];
    al = __builtin_fma(u, u, al); be = __builtin_fma(v, v, be); ga = __builtin_fma(u, v, ga);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    al += __shfl_down(al, o, 64); be += __shfl_down(be, o, 64); ga += __shfl_down(ga, o, 64);
  }
  if ((tid & 63) == 0) { red[0][tid >> 6] = al; red[1][tid >> 6] = be; red[2][tid >> 6] = ga; }
  __syncthreads();
  al = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
  be = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
  ga = (red[2][0] + red[2][1]) + (red[2][2] + red[2][3]);
  if (tid == 0) {
    gamma2[k] = ga * ga;
    if (diag2 != nullptr) diag2[k] = al * al + be * be;
  }
  if (!(fabs(ga) > 2.220446049250313e-16 * sqrt(al * be))) return;   // also alpha or beta zero, NaN
  const double zeta = (be - al) / (2.0 * ga);
  const double t = zeta == 0.0 ? 1.0 : copysign(1.0, zeta) / (fabs(zeta) + hypot(1.0, zeta));
  const double c = 1.0 / sqrt(1.0 + t * t), s = c * t;
  for (int r = tid; r < n_pad; r += 256) {
    const double u = yp[r], v = yq[r];
    yp[r] = c * u - s * v;
    yq[r] = s * u + c * v;
  }
  double* vp = Vt + static_cast<size_t>(p) * D;
  double* vq = Vt + static_cast<size_t>(q) * D;
  for (int j = tid; j < D; j += 256) {
    const double u = vp[j], v = vq[j];
    vp[j] = c * u - s * v;
    vq[j] = s * u + c * v;
  }
}

// out[0] = sum of gamma2[0 .. n_gamma), out[1] = sum of diag2[0 .. n_diag): one workgroup, every
// thread adds its strided share in order and the 256 shares are added in a fixed tree.
__global__ __launch_bounds__(256) void hestenes_sum_kernel(const double* __restrict__ gamma2, size_t n_gamma,
                                                           const double* __restrict__ diag2, int n_diag,
                                                           double* __restrict__ out) {
  __shared__ double sh[2][256];
  double g = 0.0, d = 0.0;
  for (size_t i = threadIdx.x; i < n_gamma; i += 256) g += gamma2[i];
  for (int i = threadIdx.x; i < n_diag; i += 256) d += diag2[i];
  sh[0][threadIdx.x] = g; sh[1][threadIdx.x] = d;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) { sh[0][threadIdx.x] += sh[0][threadIdx.x + w]; sh[1][threadIdx.x] += sh[1][threadIdx.x + w]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { out[0] = sh[0][0]; out[1] = sh[1][0]; }
}

// lambda_c = |y_c|^2 / n_cal
__global__ __launch_bounds__(256) void hestenes_norms_kernel(const double* __restrict__ Y, int n_pad, int n_cal,
                                                             double* __restrict__ lam) {
  __shared__ double red[4];
  const int c = blockIdx.x;
  double a = 0.0;
  for (int r = threadIdx.x; r < n_pad; r += 256) { const double u = Y[static_cast<size_t>(c) * n_pad + r]; a = __builtin_fma(u, u, a); }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a += __shfl_down(a, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) lam[c] = ((red[0] + red[1]) + (red[2] + red[3])) / static_cast<double>(n_cal);
}

static int pca_fail(hipError_t e, const char* what) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  return ROSAQ_ERR_HIP;
}

// Device part + the host bookkeeping of Eq. 4's "columns sorted by eigenvalue": descending
// order (ties keep the lower column first), negative round-off clamped to zero, each
// eigenvector signed so that its entry of largest magnitude is positive.
int pca_headwise_device(const void* X_dev, int n_cal, int D, int64_t ldx, float* Q_host,
                        double* eig_host, void* stream) {
  const int H = D / kH;
  hipStream_t st = static_cast<hipStream_t>(stream);
  double *dC = nullptr, *dV = nullptr, *dL = nullptr;
  int* dS = nullptr;
  const size_t mat = static_cast<size_t>(H) * kH * kH;
  hipError_t e = hipMalloc(&dC, mat * 8);
  if (e == hipSuccess) e = hipMalloc(&dV, mat * 8);
  if (e == hipSuccess) e = hipMalloc(&dL, static_cast<size_t>(D) * 8);
  if (e == hipSuccess) e = hipMalloc(&dS, static_cast<size_t>(H) * 4);
  std::vector<double> V, lam(D);
  std::vector<int> sweeps(H);
  const size_t lds_bytes = (static_cast<size_t>(kH) * kLd + 128 + 16) * 8 + 128 * 4;
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(jacobi128_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
  if (e == hipSuccess) {
    hipLaunchKernelGGL(second_moment_kernel, dim3(H), dim3(256), 0, st,
                       static_cast<const _Float16*>(X_dev), ldx, n_cal, dC);
    e = hipGetLastError();
  }
  if (e == hipSuccess) {
    hipLaunchKernelGGL(jacobi128_kernel, dim3(H), dim3(1024), lds_bytes, st, dC, dV, dL, dS, 1e-13, 60);
    e = hipGetLastError();
  }
  if (e == hipSuccess) {
    try { V.resize(mat); } catch (const std::bad_alloc&) { e = hipErrorOutOfMemory; }
  }
  if (e == hipSuccess) e = hipMemcpyAsync(V.data(), dV, mat * 8, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipMemcpyAsync(lam.data(), dL, static_cast<size_t>(D) * 8, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipMemcpyAsync(sweeps.data(), dS, static_cast<size_t>(H) * 4, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (dC) (void)hipFree(dC);
  if (dV) (void)hipFree(dV);
  if (dL) (void)hipFree(dL);
  if (dS) (void)hipFree(dS);
  if (e != hipSuccess) return pca_fail(e, "rosaq_pca_headwise");
  for (int h = 0; h < H; ++h)
    if (sweeps[h] < 0) {
      set_error("Jacobi did not converge within 60 sweeps (head " + std::to_string(h) + ")");
      return ROSAQ_ERR_NOCONVERGE;
    }
  for (int h = 0; h < H; ++h) {
    const double* Vh = &V[static_cast<size_t>(h) * kH * kH];
    std::vector<int> order(kH);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return lam[h * kH + a] > lam[h * kH + b]; });
    float* Qh = Q_host + static_cast<size_t>(h) * kH * kH;
    for (int j = 0; j < kH; ++j) {
      const int src = order[j];
      eig_host[h * kH + j] = std::max(lam[h * kH + src], 0.0);
      int big = 0;
      for (int i = 1; i < kH; ++i)
        if (std::fabs(Vh[i * kH + src]) > std::fabs(Vh[big * kH + src])) big = i;
      const double sign = Vh[big * kH + src] < 0.0 ? -1.0 : 1.0;
      for (int i = 0; i < kH; ++i) Qh[i * kH + j] = static_cast<float>(sign * Vh[i * kH + src]);
    }
  }
  return ROSAQ_OK;
}

// Layer-wise PCA on the device: sweeps of D - 1 rounds until the off-diagonal part of the implied
// second moment is below tol times its norm (sum gamma^2 <= tol^2 (sum lambda^2 / 2 + sum gamma^2),
// measured over a sweep), then the same host bookkeeping as the head-wise route: eigenvalues
// descending, negative round-off impossible here (norms), eigenvector signs fixed.
int pca_full_device(const void* X_dev, int n_cal, int D, int64_t ldx, float* Q_host, double* eig_host,
                    void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int n_pad = (n_cal + 3) / 4 * 4;
  const size_t pairs = static_cast<size_t>(D) / 2, rounds = static_cast<size_t>(D) - 1;
  double *dY = nullptr, *dV = nullptr, *dG = nullptr, *dD = nullptr, *dS = nullptr, *dL = nullptr;
  hipError_t e = hipMalloc(&dY, static_cast<size_t>(D) * n_pad * 8);
  if (e == hipSuccess) e = hipMalloc(&dV, static_cast<size_t>(D) * D * 8);
  if (e == hipSuccess) e = hipMalloc(&dG, rounds * pairs * 8);
  if (e == hipSuccess) e = hipMalloc(&dD, pairs * 8);
  if (e == hipSuccess) e = hipMalloc(&dS, 2 * 8);
  if (e == hipSuccess) e = hipMalloc(&dL, static_cast<size_t>(D) * 8);
  constexpr int kMaxSweeps = 60;
  constexpr double kTol = 1e-13;
  bool converged = false;
  if (e == hipSuccess) {
    hipLaunchKernelGGL(hestenes_init_kernel, dim3(D), dim3(256), 0, st, static_cast<const _Float16*>(X_dev), ldx,
                       n_cal, n_pad, D, dY, dV);
    e = hipGetLastError();
  }
  for (int sweep = 0; e == hipSuccess && sweep < kMaxSweeps && !converged; ++sweep) {
    for (size_t r = 0; r < rounds && e == hipSuccess; ++r) {
      hipLaunchKernelGGL(hestenes_round_kernel, dim3(static_cast<unsigned>(pairs)), dim3(256), 0, st, dY, dV, n_pad,
                         D, static_cast<int>(r), dG + r * pairs, r == 0 ? dD : nullptr);
      e = hipGetLastError();
    }
    if (e != hipSuccess) break;
    hipLaunchKernelGGL(hestenes_sum_kernel, dim3(1), dim3(256), 0, st, dG, rounds * pairs, dD, static_cast<int>(pairs), dS);
    e = hipGetLastError();
    double stats[2] = {0.0, 0.0};
    if (e == hipSuccess) e = hipMemcpyAsync(stats, dS, 16, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) break;
    // ||C||_F^2 n_cal^2 = sum alpha^2 + 2 sum gamma^2 at the start of the sweep; off^2 = 2 sum gamma^2
    const double off2 = 2.0 * stats[0], norm2 = stats[1] + 2.0 * stats[0];
    if (!(off2 == off2)) { e = hipErrorUnknown; break; }
    if (off2 <= kTol * kTol * norm2) converged = true;
  }
  std::vector<double> V, lam(D);
  if (e == hipSuccess) {
    hipLaunchKernelGGL(hestenes_norms_kernel, dim3(D), dim3(256), 0, st, dY, n_pad, n_cal, dL);
    e = hipGetLastError();
  }
  if (e == hipSuccess) {
    try { V.resize(static_cast<size_t>(D) * D); } catch (const std::bad_alloc&) { e = hipErrorOutOfMemory; }
  }
  if (e == hipSuccess) e = hipMemcpyAsync(V.data(), dV, static_cast<size_t>(D) * D * 8, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipMemcpyAsync(lam.data(), dL, static_cast<size_t>(D) * 8, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  for (double* q : {dY, dV, dG, dD, dS, dL})
    if (q) (void)hipFree(q);
  if (e != hipSuccess) return pca_fail(e, "rosaq_pca_full");
  if (!converged) {
    set_error("one-sided Jacobi did not converge within 60 sweeps");
    return ROSAQ_ERR_NOCONVERGE;
  }
  std::vector<int> order(D);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return lam[a] > lam[b]; });
  for (int j = 0; j < D; ++j) {
    const int src = order[j];
    const double* v = &V[static_cast<size_t>(src) * D];       // row src of Vt = eigenvector src
    eig_host[j] = std::max(lam[src], 0.0);
    int big = 0;
    for (int i = 1; i < D; ++i)
      if (std::fabs(v[i]) > std::fabs(v[big])) big = i;
    const double sign = v[big] < 0.0 ? -1.0 : 1.0;
    for (int i = 0; i < D; ++i) Q_host[static_cast<size_t>(i) * D + j] = static_cast<float>(sign * v[i]);
  }
  return ROSAQ_OK;
}

}  // namespace rosaq
