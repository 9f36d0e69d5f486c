// Cloud block of Algorithm 1 (the gradients collected on the cloud build the basis; Sec. 3.2, paragraph on guided
// perturbation sampling on the cloud): the orthonormal basis U [rows, k] of one weight matrix from its stored gradient snapshots G_1 .. G_s
// (each [rows, cols] fp32, row-major), and the gradient of the least-squares model.
//
// U spans the k-dimensional subspace of R^rows that captures the most of the snapshots (the k leading left singular
// vectors of [G_1 | ... | G_s]).  It is reached by block subspace iteration on the operator C = sum_t G_t G_t^T,
// which is never formed:
//     Y = sum_t G_t Omega              (Omega [cols, k]: the caller's seeded Gaussian start)
//     Q = orth(Y)
//     n_iter times:  T_t = G_t^T Q,  Y = sum_t G_t T_t,  Q = orth(Y)
// Each sweep reads every snapshot twice and is a pair of tall-skinny products (HBM-bound: 2 rows cols 4 bytes per
// snapshot and sweep); orth is classical Gram-Schmidt with one re-orthogonalisation per column, in one workgroup
// (rows x k with k <= 64 is at most a few MB: it lives in L2).  The subspace converges like (sigma_{k+1} / sigma_k)^(2 n):
// the caller picks n_iter for the gap it expects.  This runs every gamma rounds on the cloud, not on the client's
// step: it is written to be correct and bandwidth-shaped, not tuned.
#include "internal.h"
#include <atomic>

namespace zgr {

namespace {

constexpr int kTile = 64;      // columns (or rows) of G a block owns
constexpr int kChunk = 32;     // the other dimension, staged per step

// T[c][j] (+)= sum_r G[r][c] Q[r][j],  c < cols, j < n: G [rows, cols] (row stride ldg), Q [rows, n] (row stride ldq).
// Block = 64 columns c x 64 columns j (blockIdx.y tiles j); thread (c = tid % 64, jg = tid / 64) holds 16 values of j.
// blockIdx.z = part of the sum: rows [z row_part, (z + 1) row_part) go to T + z t_part (partial sums that sum_parts_kernel adds in order).
__global__ void __launch_bounds__(256) gt_q_kernel(const float* __restrict__ G, int64_t rows, int64_t cols, int64_t ldg, const float* __restrict__ Q, int n, int64_t ldq,
                                                   float* __restrict__ T, int64_t ldt, float scale, int accumulate, int64_t row_part, int64_t t_part) {
  __shared__ float Gs[kChunk][kTile + 1], Qs[kChunk][kTile + 1];
  const int tid = threadIdx.x, cl = tid & 63, jg = tid >> 6;
  const int64_t c0 = (int64_t)blockIdx.x * kTile;
  const int j0 = blockIdx.y * kTile;
  const int64_t r_begin = (int64_t)blockIdx.z * row_part;
  rows = rows < r_begin + row_part ? rows : r_begin + row_part;
  T += (int64_t)blockIdx.z * t_part;
  float acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  for (int64_t r0 = r_begin; r0 < rows; r0 += kChunk) {
    __syncthreads();
    for (int i = tid; i < kChunk * kTile; i += 256) {
      const int rr = i >> 6, cc = i & 63;
      const int64_t r = r0 + rr;
      Gs[rr][cc] = (r < rows && c0 + cc < cols) ? G[r * ldg + c0 + cc] : 0.f;
      Qs[rr][cc] = (r < rows && j0 + cc < n) ? Q[r * ldq + j0 + cc] : 0.f;
    }
    __syncthreads();
#pragma unroll 4
    for (int rr = 0; rr < kChunk; ++rr) {
      const float g = Gs[rr][cl];
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = __builtin_fmaf(g, Qs[rr][jg * 16 + i], acc[i]);
    }
  }
  if (c0 + cl < cols)
    for (int i = 0; i < 16; ++i) {
      const int j = j0 + jg * 16 + i;
      if (j < n) { float* t = T + (c0 + cl) * ldt + j; *t = (accumulate ? *t : 0.f) + scale * acc[i]; }
    }
}

// Y[r][j] (+)= sum_c G[r][c] T[c][j],  r < rows, j < k <= 64.  Block = 64 rows; thread (r = tid % 64, jg = tid / 64).
// blockIdx.y = part of the sum: columns [y col_part, (y + 1) col_part) go to Y + y y_part.
__global__ void __launch_bounds__(256) g_t_kernel(const float* __restrict__ G, int64_t rows, int64_t cols, const float* __restrict__ T, int k,
                                                  float* __restrict__ Y, int accumulate, int64_t col_part, int64_t y_part) {
  __shared__ float Gs[kTile][kChunk + 1], Ts[kChunk][kTile + 1];
  const int tid = threadIdx.x, rl = tid & 63, jg = tid >> 6;
  const int64_t r0 = (int64_t)blockIdx.x * kTile;
  const int64_t c_begin = (int64_t)blockIdx.y * col_part;
  const int64_t c_end = cols < c_begin + col_part ? cols : c_begin + col_part;
  Y += (int64_t)blockIdx.y * y_part;
  float acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  for (int64_t c0 = c_begin; c0 < c_end; c0 += kChunk) {
    __syncthreads();
    for (int i = tid; i < kTile * kChunk; i += 256) {
      const int rr = i >> 5, cc = i & 31;                 // consecutive threads read consecutive columns of G
      Gs[rr][cc] = (r0 + rr < rows && c0 + cc < c_end) ? G[(r0 + rr) * cols + c0 + cc] : 0.f;
    }
    for (int i = tid; i < kChunk * kTile; i += 256) {
      const int cc = i >> 6, jj = i & 63;
      Ts[cc][jj] = (c0 + cc < c_end && jj < k) ? T[(c0 + cc) * k + jj] : 0.f;
    }
    __syncthreads();
#pragma unroll 4
    for (int cc = 0; cc < kChunk; ++cc) {
      const float g = Gs[rl][cc];
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = __builtin_fmaf(g, Ts[cc][jg * 16 + i], acc[i]);
    }
  }
  if (r0 + rl < rows)
    for (int i = 0; i < 16; ++i) {
      const int j = jg * 16 + i;
      if (j < k) { float* y = Y + (r0 + rl) * k + j; *y = (accumulate ? *y : 0.f) + acc[i]; }
    }
}

// In-place orthonormalisation of the k columns of Y [rows, k] (row stride k), one workgroup of 1024 threads.
// Column j: r = Q_{<j}^T y_j, y_j -= Q_{<j} r, once more (which makes classical Gram-Schmidt as orthogonal as
// Householder for any column that is not dependent to working precision), then y_j /= ||y_j||.  Dot products are
// accumulated in fp64.  A column that the earlier ones already span (norm below 1e-6 of what it started with)
// is stored as zeros and counted in *dependent.
// IN_LDS: the block is copied into LDS first (row stride k + 1, so that threads on consecutive rows hit different banks) and
// written back at the end: the 3 k sweeps over the rows then cost LDS latency instead of L2 latency.  Same arithmetic, same order.
template <bool IN_LDS>
__global__ void __launch_bounds__(1024) orth_kernel(float* __restrict__ Yg, int64_t rows, int k, int* __restrict__ dependent) {
  __shared__ double red[16][kMaxK];
  __shared__ double coef[kMaxK];
  __shared__ int n_dep;
  extern __shared__ float orth_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ld = IN_LDS ? k + 1 : k;
  float* Y = IN_LDS ? orth_lds : Yg;
  if (IN_LDS) {
    for (int64_t i = tid; i < rows * k; i += 1024) Y[(i / k) * ld + (i % k)] = Yg[i];
    __syncthreads();
  }
  if (tid == 0) n_dep = 0;
  for (int j = 0; j < k; ++j) {
    double norm0 = 0.0;
    for (int pass = 0; pass < 3; ++pass) {
      // pass 0, 1: coefficients against the earlier columns; pass 2: the norm of what is left (slot j)
      const int n_dot = pass < 2 ? j : 1;
      for (int i0 = 0; i0 < n_dot; i0 += 8) {                      // eight dot products per sweep over the rows
        double part[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) part[i] = 0.0;
        for (int64_t r = tid; r < rows; r += 1024) {
          const float* row = Y + r * ld;
          const double yj = (double)row[j];
#pragma unroll
          for (int i = 0; i < 8; ++i)
            if (i0 + i < n_dot) part[i] += yj * (pass < 2 ? (double)row[i0 + i] : yj);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          double v = part[i];
          for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
          if (lane == 0 && i0 + i < n_dot) red[wave][i0 + i] = v;
        }
      }
      __syncthreads();
      if (tid < n_dot) {
        double v = 0.0;
        for (int w = 0; w < 16; ++w) v += red[w][tid];
        coef[tid] = v;
      }
      __syncthreads();
      if (pass < 2) {
        if (pass == 0) {                                           // remember the column's size before anything is taken out
          double n0 = 0.0;
          for (int64_t r = tid; r < rows; r += 1024) { const double y = (double)Y[r * ld + j]; n0 += y * y; }
          for (int o = 32; o > 0; o >>= 1) n0 += __shfl_xor(n0, o, 64);
          __syncthreads();
          if (lane == 0) red[wave][kMaxK - 1] = n0;
          __syncthreads();
          for (int w = 0; w < 16; ++w) norm0 += red[w][kMaxK - 1];
        }
        for (int64_t r = tid; r < rows; r += 1024) {
          float* row = Y + r * ld;
          double y = (double)row[j];
          for (int i = 0; i < j; ++i) y -= coef[i] * (double)row[i];
          row[j] = (float)y;
        }
        __syncthreads();
      } else {
        const double nrm2 = coef[0];
        const bool dep = !(nrm2 > 1e-12 * norm0) || !(nrm2 > 0.0);
        const double inv = dep ? 0.0 : 1.0 / sqrt(nrm2);
        for (int64_t r = tid; r < rows; r += 1024) Y[r * ld + j] = (float)((double)Y[r * ld + j] * inv);
        if (tid == 0 && dep) n_dep += 1;
        __syncthreads();
      }
    }
  }
  if (IN_LDS) {
    __syncthreads();
    for (int64_t i = tid; i < rows * k; i += 1024) Yg[i] = Y[(i / k) * ld + (i % k)];
  }
  if (tid == 0) *dependent = n_dep;
}

// out[i] = (accumulate ? out[i] : 0) + scale (part[0][i] + part[1][i] + ...): the parts of a split sum, added in their order
__global__ void __launch_bounds__(256) sum_parts_kernel(const float* __restrict__ part, int n_parts, int64_t stride, int64_t n, float* __restrict__ out, float scale, int accumulate) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    float v = 0.f;
    for (int z = 0; z < n_parts; ++z) v += part[(int64_t)z * stride + i];
    out[i] = (accumulate ? out[i] : 0.f) + scale * v;
  }
}

__global__ void __launch_bounds__(256) copy_basis_kernel(const float* __restrict__ Q, int64_t rows, int k, float* __restrict__ U, int ldu) {
  const int64_t n = rows * k;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) U[(i / k) * ldu + (i % k)] = Q[i];
}

// R[b][o] -= Y[b][o]  (R holds the predictions on entry)
__global__ void __launch_bounds__(256) residual_kernel(float* __restrict__ R, const float* __restrict__ Y, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) R[i] -= Y[i];
}

}  // namespace

// How many parts to split a sum over `span` terms into, so that `blocks` blocks become about one per CU-slot: at most kCloudMaxParts,
// each part a whole number of staged chunks.
static int cloud_sum_parts(int64_t blocks, int64_t span) {
  int64_t z = blocks > 0 ? 512 / blocks : 1;
  const int64_t chunks = (span + kChunk - 1) / kChunk;
  if (z > chunks) z = chunks;
  if (z > kCloudMaxParts) z = kCloudMaxParts;
  return z < 1 ? 1 : (int)z;
}

static hipError_t launch_sum_parts(const float* part, int n_parts, int64_t stride, int64_t n, float* out, float scale, int accumulate, hipStream_t s) {
  hipLaunchKernelGGL(sum_parts_kernel, dim3((unsigned)(n / 256 + 1 < 1024 ? n / 256 + 1 : 1024)), dim3(256), 0, s, part, n_parts, stride, n, out, scale, accumulate);
  return hipGetLastError();
}

// part: scratch of kCloudMaxParts * cols * n floats (ldt == n), or NULL for a single pass over all the rows
hipError_t launch_cloud_gt_q(const float* G, int64_t rows, int64_t cols, int64_t ldg, const float* Q, int n, int64_t ldq, float* T, int64_t ldt, float scale,
                             int accumulate, hipStream_t s, float* part) {
  const unsigned gx = (unsigned)((cols + kTile - 1) / kTile), gy = (unsigned)((n + kTile - 1) / kTile);
  const int z = (part && ldt == n) ? cloud_sum_parts((int64_t)gx * gy, rows) : 1;
  if (z <= 1) {
    hipLaunchKernelGGL(gt_q_kernel, dim3(gx, gy), dim3(256), 0, s, G, rows, cols, ldg, Q, n, ldq, T, ldt, scale, accumulate, rows, (int64_t)0);
    return hipGetLastError();
  }
  const int64_t chunks = (rows + kChunk - 1) / kChunk, row_part = (chunks + z - 1) / z * kChunk, stride = cols * (int64_t)n;
  hipLaunchKernelGGL(gt_q_kernel, dim3(gx, gy, (unsigned)z), dim3(256), 0, s, G, rows, cols, ldg, Q, n, ldq, part, (int64_t)n, 1.0f, 0, row_part, stride);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_sum_parts(part, z, stride, stride, T, scale, accumulate, s);
}

// part: scratch of kCloudMaxParts * rows * k floats, or NULL for a single pass over all the columns
hipError_t launch_cloud_g_t(const float* G, int64_t rows, int64_t cols, const float* T, int k, float* Y, int accumulate, hipStream_t s, float* part) {
  const unsigned gx = (unsigned)((rows + kTile - 1) / kTile);
  const int z = part ? cloud_sum_parts(gx, cols) : 1;
  if (z <= 1) {
    hipLaunchKernelGGL(g_t_kernel, dim3(gx), dim3(256), 0, s, G, rows, cols, T, k, Y, accumulate, cols, (int64_t)0);
    return hipGetLastError();
  }
  const int64_t chunks = (cols + kChunk - 1) / kChunk, col_part = (chunks + z - 1) / z * kChunk, stride = rows * (int64_t)k;
  hipLaunchKernelGGL(g_t_kernel, dim3(gx, (unsigned)z), dim3(256), 0, s, G, rows, cols, T, k, part, 0, col_part, stride);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_sum_parts(part, z, stride, stride, Y, 1.0f, accumulate, s);
}

hipError_t launch_cloud_orth(float* Y, int64_t rows, int k, int* dependent, hipStream_t s) {
  // the block in LDS when it fits beside the kernel's own 9 KB (rows (k + 1) floats: 2048 x 16 does, 8192 x 16 does not)
  const size_t lds = (size_t)rows * (size_t)(k + 1) * sizeof(float);
  if (lds <= 144 * 1024) {
    static std::atomic<bool> attr_set{false};              // set twice by racing threads at worst: the call is idempotent
    if (!attr_set) {
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(orth_kernel<true>), hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    hipLaunchKernelGGL(orth_kernel<true>, dim3(1), dim3(1024), lds, s, Y, rows, k, dependent);
  } else {
    hipLaunchKernelGGL(orth_kernel<false>, dim3(1), dim3(1024), 0, s, Y, rows, k, dependent);
  }
  return hipGetLastError();
}

hipError_t launch_cloud_copy_basis(const float* Q, int64_t rows, int k, float* U, int ldu, hipStream_t s) {
  const int64_t n = rows * k;
  hipLaunchKernelGGL(copy_basis_kernel, dim3((unsigned)(n / 256 + 1 < 1024 ? n / 256 + 1 : 1024)), dim3(256), 0, s, Q, rows, k, U, ldu);
  return hipGetLastError();
}

hipError_t launch_cloud_residual(float* R, const float* Y, int64_t n, hipStream_t s) {
  hipLaunchKernelGGL(residual_kernel, dim3((unsigned)(n / 256 + 1 < 1024 ? n / 256 + 1 : 1024)), dim3(256), 0, s, R, Y, n);
  return hipGetLastError();
}

}  // namespace zgr
