// PCA of the calibration activations on the GPU (Sec. 3.1 Eq. 4; per attention head Sec. 3.1.1,
// Eq. 6): the eigenvectors of C = X^T X / n_cal are the right singular vectors of X, its
// eigenvalues the squared column norms of X V / n_cal.  One-sided Jacobi: plane rotations are
// applied to pairs of columns of X (kept transposed, Y[c][:] = column c, so that a column is
// contiguous) until all columns are mutually orthogonal; the same rotations accumulate in V.
// C itself is never formed, and a rotation touches two rows of Y and of V only, so the disjoint
// pairs of a round run on one workgroup each with no exchange at all -- one launch per round,
// Db - 1 rounds per sweep.  A layer-wise rotation is one problem of dimension D; a head-wise one
// is D / 128 independent problems of dimension 128 that share every launch.
// Calibration-time code: it allocates its own scratch and waits for the result.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <numeric>
#include <string>
#include <vector>

#include "rosaq_internal.h"

namespace rosaq {

// Y[c][r] = X[r][c] in fp64 (rows padded with zeros to n_pad); Vt of every block = I
// (Vt[c][j], c the global channel, j the channel inside c's block of Db).
__global__ __launch_bounds__(256) void hestenes_init_kernel(const _Float16* __restrict__ X, int64_t ldx,
                                                            int n_cal, int n_pad, int Db,
                                                            double* __restrict__ Y, double* __restrict__ Vt) {
  const int c = blockIdx.x;
  for (int r = threadIdx.x; r < n_pad; r += 256)
    Y[static_cast<size_t>(c) * n_pad + r] = r < n_cal ? static_cast<double>(X[static_cast<int64_t>(r) * ldx + c]) : 0.0;
  for (int j = threadIdx.x; j < Db; j += 256) Vt[static_cast<size_t>(c) * Db + j] = j == c % Db ? 1.0 : 0.0;
}

// One round: workgroup (block b, seat k) rotates the pair (p, q) that the round-robin tournament
// assigns to seat k (player Db - 1 stays, the others move one seat per round; seat k meets seat
// Db - 1 - k).
//   alpha = |y_p|^2, beta = |y_q|^2, gamma = y_p . y_q;  zeta = (beta - alpha) / (2 gamma),
//   t = sign(zeta) / (|zeta| + sqrt(1 + zeta^2)), c = 1 / sqrt(1 + t^2), s = c t,
//   (y_p, y_q) <- (c y_p - s y_q, s y_p + c y_q), the same for the rows p, q of Vt.
// Pairs that are orthogonal to round-off (|gamma| <= eps sqrt(alpha beta)) are left alone.
// gamma^2 of every pair (before its rotation) and, in the first round of a sweep, alpha^2 + beta^2
// go to slots that a later launch adds up in a fixed order.
__global__ __launch_bounds__(256) void hestenes_round_kernel(double* __restrict__ Y, double* __restrict__ Vt,
                                                             int n_pad, int Db, int round,
                                                             double* __restrict__ gamma2,
                                                             double* __restrict__ diag2) {
  __shared__ double red[3][4];
  const int half = Db / 2;
  const int blk = blockIdx.x / half, k = blockIdx.x - blk * half, tid = threadIdx.x;
  auto player = [&](int seat) { return seat == Db - 1 ? Db - 1 : (seat + round) % (Db - 1); };
  const int a = player(k), b = player(Db - 1 - k);
  const size_t p = static_cast<size_t>(blk) * Db + (a < b ? a : b), q = static_cast<size_t>(blk) * Db + (a < b ? b : a);
  double* yp = Y + p * n_pad;
  double* yq = Y + q * n_pad;
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
    gamma2[blockIdx.x] = ga * ga;
    if (diag2 != nullptr) diag2[blockIdx.x] = al * al + be * be;
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
  double* vp = Vt + p * Db;
  double* vq = Vt + q * Db;
  for (int j = tid; j < Db; j += 256) {
    const double u = vp[j], v = vq[j];
    vp[j] = c * u - s * v;
    vq[j] = s * u + c * v;
  }
}

// Per block b: out[2 b] = sum over rounds and seats of gamma2, out[2 b + 1] = sum over seats of
// diag2.  One workgroup per block; every thread adds its strided share in order and the 256
// shares are added in a fixed tree, so the sums do not depend on scheduling.
__global__ __launch_bounds__(256) void hestenes_sum_kernel(const double* __restrict__ gamma2, int rounds,
                                                           const double* __restrict__ diag2, int half,
                                                           int seats_total, double* __restrict__ out) {
  __shared__ double sh[2][256];
  const int blk = blockIdx.x;
  double g = 0.0, d = 0.0;
  for (int i = threadIdx.x; i < rounds * half; i += 256)
    g += gamma2[static_cast<size_t>(i / half) * seats_total + blk * half + i % half];
  for (int i = threadIdx.x; i < half; i += 256) d += diag2[blk * half + i];
  sh[0][threadIdx.x] = g; sh[1][threadIdx.x] = d;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) { sh[0][threadIdx.x] += sh[0][threadIdx.x + w]; sh[1][threadIdx.x] += sh[1][threadIdx.x + w]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { out[2 * blk] = sh[0][0]; out[2 * blk + 1] = sh[1][0]; }
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

// D / Db independent PCA problems of dimension Db on the channels [b Db, (b + 1) Db): sweeps of
// Db - 1 rounds until, in every block, the off-diagonal part of the implied second moment is below
// tol times its norm (2 sum gamma^2 <= tol^2 (sum alpha^2 + 2 sum gamma^2), measured over a
// sweep).  Then the host bookkeeping of Eq. 4's "columns sorted by eigenvalue" per block:
// descending order (ties keep the lower column first), each eigenvector signed so that its entry
// of largest magnitude is positive.  Q_host is [D / Db][Db][Db], block b holding its eigenvectors
// as columns (for Db = D that is the row-major D x D rotation).
static int pca_blocks_device(const void* X_dev, int n_cal, int D, int Db, int64_t ldx, float* Q_host,
                             double* eig_host, void* stream, const char* who) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int n_pad = (n_cal + 3) / 4 * 4, blocks = D / Db, half = Db / 2, rounds = Db - 1;
  const int seats = blocks * half;
  // host bookkeeping first: if it cannot be had, nothing on the device has been allocated yet
  std::vector<double> stats(static_cast<size_t>(blocks) * 2), V, lam(D);
  std::vector<int> order(Db);
  double *dY = nullptr, *dV = nullptr, *dG = nullptr, *dD = nullptr, *dS = nullptr, *dL = nullptr;
  hipError_t e = hipMalloc(&dY, static_cast<size_t>(D) * n_pad * 8);
  if (e == hipSuccess) e = hipMalloc(&dV, static_cast<size_t>(D) * Db * 8);
  if (e == hipSuccess) e = hipMalloc(&dG, static_cast<size_t>(rounds) * seats * 8);
  if (e == hipSuccess) e = hipMalloc(&dD, static_cast<size_t>(seats) * 8);
  if (e == hipSuccess) e = hipMalloc(&dS, static_cast<size_t>(blocks) * 2 * 8);
  if (e == hipSuccess) e = hipMalloc(&dL, static_cast<size_t>(D) * 8);
  constexpr int kMaxSweeps = 60;
  constexpr double kTol = 1e-13;
  bool converged = false;
  if (e == hipSuccess) {
    hipLaunchKernelGGL(hestenes_init_kernel, dim3(D), dim3(256), 0, st, static_cast<const _Float16*>(X_dev), ldx,
                       n_cal, n_pad, Db, dY, dV);
    e = hipGetLastError();
  }
  for (int sweep = 0; e == hipSuccess && sweep < kMaxSweeps && !converged; ++sweep) {
    for (int r = 0; r < rounds && e == hipSuccess; ++r) {
      hipLaunchKernelGGL(hestenes_round_kernel, dim3(seats), dim3(256), 0, st, dY, dV, n_pad, Db, r,
                         dG + static_cast<size_t>(r) * seats, r == 0 ? dD : nullptr);
      e = hipGetLastError();
    }
    if (e != hipSuccess) break;
    hipLaunchKernelGGL(hestenes_sum_kernel, dim3(blocks), dim3(256), 0, st, dG, rounds, dD, half, seats, dS);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(stats.data(), dS, stats.size() * 8, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) break;
    converged = true;
    for (int b = 0; b < blocks; ++b) {
      // ||C_b||_F^2 n_cal^2 = sum alpha^2 + 2 sum gamma^2 at the start of the sweep; off^2 = 2 sum gamma^2
      const double off2 = 2.0 * stats[2 * b], norm2 = stats[2 * b + 1] + 2.0 * stats[2 * b];
      if (!(off2 == off2)) { e = hipErrorUnknown; break; }
      if (!(off2 <= kTol * kTol * norm2)) converged = false;
    }
  }
  if (e == hipSuccess) {
    hipLaunchKernelGGL(hestenes_norms_kernel, dim3(D), dim3(256), 0, st, dY, n_pad, n_cal, dL);
    e = hipGetLastError();
  }
  if (e == hipSuccess) {
    try { V.resize(static_cast<size_t>(D) * Db); } catch (const std::bad_alloc&) { e = hipErrorOutOfMemory; }
  }
  if (e == hipSuccess) e = hipMemcpyAsync(V.data(), dV, static_cast<size_t>(D) * Db * 8, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipMemcpyAsync(lam.data(), dL, static_cast<size_t>(D) * 8, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  for (double* q : {dY, dV, dG, dD, dS, dL})
    if (q) (void)hipFree(q);
  if (e != hipSuccess) return pca_fail(e, who);
  if (!converged) {
    set_error("one-sided Jacobi did not converge within 60 sweeps");
    return ROSAQ_ERR_NOCONVERGE;
  }
  for (int b = 0; b < blocks; ++b) {
    const double* lb = &lam[static_cast<size_t>(b) * Db];
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return lb[x] > lb[y]; });
    float* Qb = Q_host + static_cast<size_t>(b) * Db * Db;
    for (int j = 0; j < Db; ++j) {
      const int src = order[j];
      const double* v = &V[(static_cast<size_t>(b) * Db + src) * Db];    // row src of Vt = eigenvector src
      eig_host[static_cast<size_t>(b) * Db + j] = std::max(lb[src], 0.0);
      int big = 0;
      for (int i = 1; i < Db; ++i)
        if (std::fabs(v[i]) > std::fabs(v[big])) big = i;
      const double sign = v[big] < 0.0 ? -1.0 : 1.0;
      for (int i = 0; i < Db; ++i) Qb[static_cast<size_t>(i) * Db + j] = static_cast<float>(sign * v[i]);
    }
  }
  return ROSAQ_OK;
}

int pca_headwise_device(const void* X_dev, int n_cal, int D, int64_t ldx, float* Q_host,
                        double* eig_host, void* stream) {
  return pca_blocks_device(X_dev, n_cal, D, kHeadDim, ldx, Q_host, eig_host, stream, "rosaq_pca_headwise");
}

int pca_full_device(const void* X_dev, int n_cal, int D, int64_t ldx, float* Q_host, double* eig_host,
                    void* stream) {
  return pca_blocks_device(X_dev, n_cal, D, D, ldx, Q_host, eig_host, stream, "rosaq_pca_full");
}

}  // namespace rosaq
