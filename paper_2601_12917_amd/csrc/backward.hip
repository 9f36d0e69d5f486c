// Backward pass of the cloud block of Algorithm 1 (back-propagation on the public dataset with the current weights,
// whose gradients build the basis; Sec. 3.2, paragraph on guided perturbation sampling on the cloud): dL/dtheta of the loss of forward.hip, by the chain rule
// layer by layer, in fp32.  The forward pass that precedes it runs the client's own kernels and keeps every layer's
// intermediate results; these kernels take them back in reverse order.
//
// This runs on the cloud once per stored gradient snapshot, not on the client's step: the kernels are plain
// (LDS-tiled fp32 products with general strides, one workgroup per row for the row-wise rules), deterministic (no
// atomics: every sum has a fixed order) and not tuned.
#include "backward.h"

namespace zgr {

namespace {

struct bf16_t { uint16_t bits; };
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float((uint32_t)x.bits << 16); }
__device__ __forceinline__ void from_f32(float x, float& o) { o = x; }
__device__ __forceinline__ void from_f32(float x, bf16_t& o) {
  const __bf16 h = static_cast<__bf16>(x);
  o.bits = __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// block of 256 threads
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// ------------------------------------------------------------------ C (+)= alpha A B with general strides
// C[i][j] = sum_k A[i ars + k acs] B[k brs + j bcs], i < M, j < N, k < K; A and B fp32 (a gradient) or the storage
// type (a weight or a kept activation).  64 x 64 tile, 16 deep, 4 x 4 outputs per thread; every output adds its K terms
// in the order of k.  The two uses on weights:
//   input gradient   dA [M, K'] = dY [M, N'] W [N', K']      : A = dY (ars = N', acs = 1), B = W  (brs = K', bcs = 1)
//   weight gradient  dW [N', K'] = dY^T [N', M] A_in [M, K'] : A = dY (ars = 1, acs = N'), B = A_in (brs = K', bcs = 1)
// Batched over blockIdx.z = z: operand X of batch z starts at X + (z / zdiv) * x_outer + (z % zdiv) * x_inner (elements).
struct BatchOffsets { int zdiv; int64_t a_outer, a_inner, b_outer, b_inner, c_outer, c_inner; };

template <typename TA, typename TB>
__global__ void __launch_bounds__(256) gemm_strided_kernel(const TA* __restrict__ A, int64_t ars, int64_t acs, const TB* __restrict__ B, int64_t brs, int64_t bcs,
                                                           float* __restrict__ C, int64_t ldc, int M, int N, int K, float alpha, int accumulate, BatchOffsets bo) {
  __shared__ float As[16][64 + 4], Bs[16][64 + 4];
  {
    const int zo = (int)blockIdx.z / bo.zdiv, zi = (int)blockIdx.z % bo.zdiv;
    A += zo * bo.a_outer + zi * bo.a_inner;
    B += zo * bo.b_outer + zi * bo.b_inner;
    C += zo * bo.c_outer + zi * bo.c_inner;
  }
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const bool a_rows_contig = ars == 1, b_k_contig = brs == 1;       // which index consecutive threads should walk
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      const int ra = a_rows_contig ? (i & 63) : (i >> 4), ka = a_rows_contig ? (i >> 6) : (i & 15);
      As[ka][ra] = (m0 + ra < M && k0 + ka < K) ? to_f32(A[(int64_t)(m0 + ra) * ars + (int64_t)(k0 + ka) * acs]) : 0.f;
      const int cb = b_k_contig ? (i >> 4) : (i & 63), kb = b_k_contig ? (i & 15) : (i >> 6);
      Bs[kb][cb] = (n0 + cb < N && k0 + kb < K) ? to_f32(B[(int64_t)(k0 + kb) * brs + (int64_t)(n0 + cb) * bcs]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) { float* c = C + (int64_t)m * ldc + n; *c = (accumulate ? *c : 0.f) + alpha * acc[i][j]; }
    }
}

// ------------------------------------------------------------------ operands for the matrix-core products (bf16 models)
// The bf16 GEMM of the forward pass computes A W^T with both operands contiguous along the contraction.  A backward
// product contracts over another index, so its operands are first written out in bf16 with that index innermost:
//   out[c][r] = in[r][c]   (transpose, 64 x 64 tiles through LDS)      or      out[r][c] = in[r][c]   (rounding only)
// Elements [rows, ld_out) of every output row (transpose) and [cols, ld_out) (rounding) are written as zeros: padding of the
// contraction up to the multiple of 64 the GEMM asks for.
template <typename TIN>
__global__ void __launch_bounds__(256) transpose_bf16_kernel(const TIN* __restrict__ in, int rows, int cols, int64_t ld_in, bf16_t* __restrict__ out, int64_t ld_out) {
  __shared__ float tile[64][65];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int r = i >> 6, c = i & 63;
    tile[r][c] = (r0 + r < rows && c0 + c < cols) ? to_f32(in[(int64_t)(r0 + r) * ld_in + c0 + c]) : 0.f;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int c = i >> 6, r = i & 63;
    if (r0 + r < ld_out && c0 + c < cols) from_f32(tile[r][c], out[(int64_t)(c0 + c) * ld_out + r0 + r]);      // tile holds zeros past `rows`
  }
}
__global__ void __launch_bounds__(256) round_bf16_kernel(const float* __restrict__ in, int rows, int cols, int64_t ld_in, bf16_t* __restrict__ out, int64_t ld_out) {
  const int64_t n = (int64_t)rows * ld_out;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / ld_out, c = i % ld_out;
    from_f32(c < cols ? in[r * ld_in + c] : 0.f, out[i]);
  }
}

// out[n] = sum_m Y[m ld + n]  (bias gradients), in two stages with a fixed shape so that the order of the additions
// never depends on scheduling: kColParts row chunks are summed side by side (64 columns per block, 4 row groups),
// then the chunk sums are added in chunk order.
constexpr int kColParts = 64;
__global__ void __launch_bounds__(256) colsum_partial_kernel(const float* __restrict__ Y, int M, int N, int64_t ld, float* __restrict__ part) {
  __shared__ float acc[4][64];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63), g = threadIdx.x >> 6;
  const int chunk = (M + kColParts - 1) / kColParts;
  const int m_begin = blockIdx.y * chunk, m_end = min(M, m_begin + chunk);
  float s = 0.f;
  if (c < N)
    for (int m = m_begin + g; m < m_end; m += 4) s += Y[(int64_t)m * ld + c];
  acc[g][threadIdx.x & 63] = s;
  __syncthreads();
  if (g == 0 && c < N) part[(size_t)blockIdx.y * N + c] = (acc[0][threadIdx.x] + acc[1][threadIdx.x]) + (acc[2][threadIdx.x] + acc[3][threadIdx.x]);
}
__global__ void __launch_bounds__(256) colsum_final_kernel(const float* __restrict__ part, int N, float* __restrict__ out) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= N) return;
  float s = 0.f;
  for (int p = 0; p < kColParts; ++p) s += part[(size_t)p * N + c];
  out[c] = s;
}

__global__ void __launch_bounds__(256) fill_kernel(float* __restrict__ p, int64_t n, float v) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = v;
}

// ------------------------------------------------------------------ softmax cross-entropy
// In place on a row of logits: d = (softmax - onehot(target)) * inv_count, or zeros for a row without a target.
__global__ void __launch_bounds__(256) ce_backward_kernel(float* __restrict__ logits, const int32_t* __restrict__ targets, int n, float inv_count) {
  __shared__ float red[4];
  float* row = logits + (size_t)blockIdx.x * n;
  const int tgt = targets[blockIdx.x];
  if (tgt < 0 || tgt >= n) {                        // uniform over the block
    for (int i = threadIdx.x; i < n; i += 256) row[i] = 0.f;
    return;
  }
  float mx = -INFINITY;
  for (int i = threadIdx.x; i < n; i += 256) mx = fmaxf(mx, row[i]);
  mx = block_max(mx, red);
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += expf(row[i] - mx);
  s = block_sum(s, red);
  const float inv = 1.0f / s;
  for (int i = threadIdx.x; i < n; i += 256) row[i] = (expf(row[i] - mx) * inv - (i == tgt ? 1.0f : 0.f)) * inv_count;
}

// ------------------------------------------------------------------ LayerNorm
// y = xhat g + b, xhat = (x - mu) rstd.  Per row: dx = rstd (dy g - mean(dy g) - xhat mean(dy g xhat)), written as
// dx_out = (add ? add : 0) + dx (dx_out may be add or dy itself: every sum over the row is taken before the row is
// written, and an element is written by the thread that read it).
template <typename T>
__global__ void __launch_bounds__(256) ln_backward_kernel(const float* __restrict__ x, const T* __restrict__ g, const float* dy,
                                                          const float* add, float* dx_out, int d, float eps) {   // add or dy may be dx_out
  __shared__ float red[4];
  const size_t o = (size_t)blockIdx.x * d;
  const float* row = x + o;
  const float* drow = dy + o;
  float s = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) s += row[i];
  const float mu = block_sum(s, red) / d;
  float v = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) { const float t = row[i] - mu; v += t * t; }
  const float rstd = 1.0f / sqrtf(block_sum(v, red) / d + eps);
  float s1 = 0.f, s2 = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float dg = drow[i] * to_f32(g[i]);
    s1 += dg;
    s2 += dg * ((row[i] - mu) * rstd);
  }
  s1 = block_sum(s1, red) / d;
  s2 = block_sum(s2, red) / d;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float xhat = (row[i] - mu) * rstd;
    const float r = rstd * (drow[i] * to_f32(g[i]) - s1 - xhat * s2);
    dx_out[o + i] = (add ? add[o + i] : 0.f) + r;
  }
}

// (mu, rstd) of every row, for the parameter gradients
__global__ void __launch_bounds__(256) ln_stats_kernel(const float* __restrict__ x, float* __restrict__ stats, int d, float eps) {
  __shared__ float red[4];
  const float* row = x + (size_t)blockIdx.x * d;
  float s = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) s += row[i];
  const float mu = block_sum(s, red) / d;
  float v = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) { const float t = row[i] - mu; v += t * t; }
  const float rstd = 1.0f / sqrtf(block_sum(v, red) / d + eps);
  if (threadIdx.x == 0) { stats[2 * blockIdx.x] = mu; stats[2 * blockIdx.x + 1] = rstd; }
}

// dg[c] = sum_m dy[m][c] xhat[m][c], db[c] = sum_m dy[m][c]: chunk sums as above (part: [2][kColParts][d]), then
// colsum_final_kernel on each half
__global__ void __launch_bounds__(256) ln_param_grad_partial_kernel(const float* __restrict__ x, const float* __restrict__ dy, const float* __restrict__ stats,
                                                                    int M, int d, float* __restrict__ part) {
  __shared__ float pg[4][64], pb[4][64];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63), grp = threadIdx.x >> 6;
  const int chunk = (M + kColParts - 1) / kColParts;
  const int m_begin = blockIdx.y * chunk, m_end = min(M, m_begin + chunk);
  float sg = 0.f, sb = 0.f;
  if (c < d)
    for (int m = m_begin + grp; m < m_end; m += 4) {
      const float dyv = dy[(size_t)m * d + c];
      sg += dyv * ((x[(size_t)m * d + c] - stats[2 * m]) * stats[2 * m + 1]);
      sb += dyv;
    }
  pg[grp][threadIdx.x & 63] = sg; pb[grp][threadIdx.x & 63] = sb;
  __syncthreads();
  if (grp == 0 && c < d) {
    part[(size_t)blockIdx.y * d + c] = (pg[0][threadIdx.x] + pg[1][threadIdx.x]) + (pg[2][threadIdx.x] + pg[3][threadIdx.x]);
    part[(size_t)(kColParts + blockIdx.y) * d + c] = (pb[0][threadIdx.x] + pb[1][threadIdx.x]) + (pb[2][threadIdx.x] + pb[3][threadIdx.x]);
  }
}

// ------------------------------------------------------------------ feed-forward activation: erf-GELU or ReLU
template <typename T, bool RELU>
__global__ void __launch_bounds__(256) act_forward_kernel(const float* __restrict__ u, T* __restrict__ f, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const float x = u[i];
    from_f32(RELU ? fmaxf(x, 0.f) : 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)), f[i]);
  }
}
// du = df * act'(u), in place on df: GELU' = Phi(u) + u phi(u), ReLU' = [u > 0]
template <bool RELU>
__global__ void __launch_bounds__(256) act_backward_kernel(const float* __restrict__ u, float* __restrict__ df, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const float x = u[i];
    if (RELU) { if (!(x > 0.f)) df[i] = 0.f; continue; }
    const float cdf = 0.5f * (1.0f + erff(x * 0.70710678118654752f));
    const float pdf = 0.3989422804014327f * expf(-0.5f * x * x);
    df[i] *= cdf + x * pdf;
  }
}

__global__ void __launch_bounds__(256) add_kernel(float* __restrict__ dst, const float* __restrict__ src, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) dst[i] += src[i];
}

// ------------------------------------------------------------------ attention
// qkv [B T, 3 d]: query, key, value of head h at columns h dh, d + h dh, 2 d + h dh.  Key j takes part in query i's
// softmax when j < length (the sequence's length, or T) and, under the causal mask, j <= i.
// Five batched products per head and one row-wise rule between them:
//   S = Q K^T / sqrt dh and dP = dctx V^T             (into the P and dS buffers)
//   p = softmax(S) over the visible keys, ds = p (dP - p . dP), zeros at masked keys        (attn_backward_rows_kernel, in place)
//   dQ = dS K / sqrt dh,   dK = dS^T Q / sqrt dh,   dV = P^T dctx
// One block per row (b, h, i) of the two [T, T] buffers; a thread holds up to MAXJ of the row's entries (T <= 256 MAXJ).
__global__ void __launch_bounds__(256) attn_backward_rows_kernel(const int32_t* __restrict__ lengths, int seq, int n_head, int causal,
                                                                 float* __restrict__ P, float* __restrict__ dS) {
  __shared__ float red[4];
  const int i = blockIdx.x % seq, b = blockIdx.x / (seq * n_head);
  int kend = lengths ? lengths[b] : seq;
  kend = kend < seq ? kend : seq;
  if (causal) kend = kend < i + 1 ? kend : i + 1;
  float* prow = P + (size_t)blockIdx.x * seq;
  float* srow = dS + (size_t)blockIdx.x * seq;
  constexpr int MAXJ = kBackwardMaxSeq / 256;
  float sc[MAXJ], dp[MAXJ];
  float mx = -INFINITY;
#pragma unroll
  for (int u = 0; u < MAXJ; ++u) {
    const int j = threadIdx.x + 256 * u;
    sc[u] = -INFINITY; dp[u] = 0.f;
    if (j < kend) { sc[u] = prow[j]; dp[u] = srow[j]; mx = fmaxf(mx, sc[u]); }
  }
  mx = block_max(mx, red);
  float den = 0.f;
#pragma unroll
  for (int u = 0; u < MAXJ; ++u) { sc[u] = (threadIdx.x + 256 * u < kend) ? expf(sc[u] - mx) : 0.f; den += sc[u]; }
  den = block_sum(den, red);
  const float inv = den > 0.f ? 1.0f / den : 0.f;
  float dot = 0.f;
#pragma unroll
  for (int u = 0; u < MAXJ; ++u) { sc[u] *= inv; dot += sc[u] * dp[u]; }
  dot = block_sum(dot, red);
#pragma unroll
  for (int u = 0; u < MAXJ; ++u) {
    const int j = threadIdx.x + 256 * u;
    if (j < seq) { prow[j] = sc[u]; srow[j] = sc[u] * (dp[u] - dot); }
  }
}

// ------------------------------------------------------------------ embeddings
// x0[m] = E[tok[m]] + Pe[m mod seq]: one thread per column walks the rows in order (tokens repeat, so the adds into
// one row of dE must be ordered to be reproducible); dE accumulates (the tied head has written it), dPe is overwritten.
__global__ void __launch_bounds__(256) embed_backward_kernel(const int32_t* __restrict__ tok, const float* __restrict__ dx, int M, int seq, int d, int vocab,
                                                             float* __restrict__ dE, float* __restrict__ dPe, int max_pos) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d) return;
  for (int p = 0; p < max_pos; ++p) dPe[(size_t)p * d + c] = 0.f;
  for (int m = 0; m < M; ++m) {
    int t = tok[m];
    t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
    const float g = dx[(size_t)m * d + c];
    dE[(size_t)t * d + c] += g;
    dPe[(size_t)(m % seq) * d + c] += g;
  }
}

}  // namespace

static unsigned grid_1d(int64_t n) { const int64_t b = (n + 255) / 256; return (unsigned)(b < 1 ? 1 : (b > 4096 ? 4096 : b)); }

template <typename TA>
static hipError_t launch_bw_gemm_batched(const TA* A, int64_t ars, int64_t acs, int b_dtype, const void* B, int64_t brs, int64_t bcs, float* C, int64_t ldc,
                                         int M, int N, int K, float alpha, int accumulate, int batches, const BatchOffsets& bo, hipStream_t s) {
  if (M < 1 || N < 1 || batches < 1) return hipSuccess;
  if (batches > 65535 || (M + 63) / 64 > 65535) return hipErrorInvalidValue;
  const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64), (unsigned)batches);
  if (b_dtype == 1) hipLaunchKernelGGL((gemm_strided_kernel<TA, bf16_t>), grid, dim3(256), 0, s, A, ars, acs, reinterpret_cast<const bf16_t*>(B), brs, bcs, C, ldc, M, N, K, alpha, accumulate, bo);
  else              hipLaunchKernelGGL((gemm_strided_kernel<TA, float>), grid, dim3(256), 0, s, A, ars, acs, reinterpret_cast<const float*>(B), brs, bcs, C, ldc, M, N, K, alpha, accumulate, bo);
  return hipGetLastError();
}

hipError_t launch_bw_gemm(int b_dtype, const float* A, int64_t ars, int64_t acs, const void* B, int64_t brs, int64_t bcs, float* C, int64_t ldc,
                          int M, int N, int K, float alpha, int accumulate, hipStream_t s) {
  return launch_bw_gemm_batched(A, ars, acs, b_dtype, B, brs, bcs, C, ldc, M, N, K, alpha, accumulate, 1, BatchOffsets{1, 0, 0, 0, 0, 0, 0}, s);
}

hipError_t launch_bw_transpose_bf16(int in_dtype, const void* in, int rows, int cols, int64_t ld_in, void* out, int64_t ld_out, hipStream_t s) {
  if (rows < 1 || cols < 1) return hipSuccess;
  const dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((ld_out + 63) / 64));
  if (in_dtype == 1) hipLaunchKernelGGL(transpose_bf16_kernel<bf16_t>, grid, dim3(256), 0, s, reinterpret_cast<const bf16_t*>(in), rows, cols, ld_in, reinterpret_cast<bf16_t*>(out), ld_out);
  else               hipLaunchKernelGGL(transpose_bf16_kernel<float>, grid, dim3(256), 0, s, reinterpret_cast<const float*>(in), rows, cols, ld_in, reinterpret_cast<bf16_t*>(out), ld_out);
  return hipGetLastError();
}

hipError_t launch_bw_round_bf16(const float* in, int rows, int cols, int64_t ld_in, void* out, int64_t ld_out, hipStream_t s) {
  if (rows < 1 || cols < 1) return hipSuccess;
  hipLaunchKernelGGL(round_bf16_kernel, dim3(grid_1d((int64_t)rows * ld_out)), dim3(256), 0, s, in, rows, cols, ld_in, reinterpret_cast<bf16_t*>(out), ld_out);
  return hipGetLastError();
}

size_t bw_colsum_scratch_floats(int n_max) { return (size_t)2 * kColParts * (size_t)n_max; }

hipError_t launch_bw_colsum(const float* Y, int M, int N, int64_t ld, float* out, float* part, hipStream_t s) {
  hipLaunchKernelGGL(colsum_partial_kernel, dim3((unsigned)((N + 63) / 64), kColParts), dim3(256), 0, s, Y, M, N, ld, part);
  hipLaunchKernelGGL(colsum_final_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, s, part, N, out);
  return hipGetLastError();
}

hipError_t launch_bw_fill(float* p, int64_t n, float v, hipStream_t s) {
  if (n < 1) return hipSuccess;
  hipLaunchKernelGGL(fill_kernel, dim3(grid_1d(n)), dim3(256), 0, s, p, n, v);
  return hipGetLastError();
}

hipError_t launch_bw_cross_entropy(float* logits, const int32_t* targets, int rows, int n, float inv_count, hipStream_t s) {
  hipLaunchKernelGGL(ce_backward_kernel, dim3((unsigned)rows), dim3(256), 0, s, logits, targets, n, inv_count);
  return hipGetLastError();
}

hipError_t launch_bw_layernorm(int dtype, const float* x, const void* g, const float* dy, const float* add, float* dx_out, float* stats, float* dg, float* db,
                               float* part, int M, int d, float eps, hipStream_t s) {
  // the parameter gradients read dy: they go first, so that dx_out may overwrite it
  hipLaunchKernelGGL(ln_stats_kernel, dim3((unsigned)M), dim3(256), 0, s, x, stats, d, eps);
  hipLaunchKernelGGL(ln_param_grad_partial_kernel, dim3((unsigned)((d + 63) / 64), kColParts), dim3(256), 0, s, x, dy, stats, M, d, part);
  hipLaunchKernelGGL(colsum_final_kernel, dim3((unsigned)((d + 255) / 256)), dim3(256), 0, s, part, d, dg);
  hipLaunchKernelGGL(colsum_final_kernel, dim3((unsigned)((d + 255) / 256)), dim3(256), 0, s, part + (size_t)kColParts * d, d, db);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (dtype == 1) hipLaunchKernelGGL(ln_backward_kernel<bf16_t>, dim3((unsigned)M), dim3(256), 0, s, x, reinterpret_cast<const bf16_t*>(g), dy, add, dx_out, d, eps);
  else            hipLaunchKernelGGL(ln_backward_kernel<float>, dim3((unsigned)M), dim3(256), 0, s, x, reinterpret_cast<const float*>(g), dy, add, dx_out, d, eps);
  return hipGetLastError();
}

hipError_t launch_bw_act_forward(int dtype, int relu, const float* u, void* f, int64_t n, hipStream_t s) {
  const dim3 grid(grid_1d(n));
  if (dtype == 1) {
    if (relu) hipLaunchKernelGGL((act_forward_kernel<bf16_t, true>), grid, dim3(256), 0, s, u, reinterpret_cast<bf16_t*>(f), n);
    else      hipLaunchKernelGGL((act_forward_kernel<bf16_t, false>), grid, dim3(256), 0, s, u, reinterpret_cast<bf16_t*>(f), n);
  } else {
    if (relu) hipLaunchKernelGGL((act_forward_kernel<float, true>), grid, dim3(256), 0, s, u, reinterpret_cast<float*>(f), n);
    else      hipLaunchKernelGGL((act_forward_kernel<float, false>), grid, dim3(256), 0, s, u, reinterpret_cast<float*>(f), n);
  }
  return hipGetLastError();
}

hipError_t launch_bw_act(int relu, const float* u, float* df, int64_t n, hipStream_t s) {
  if (relu) hipLaunchKernelGGL(act_backward_kernel<true>, dim3(grid_1d(n)), dim3(256), 0, s, u, df, n);
  else      hipLaunchKernelGGL(act_backward_kernel<false>, dim3(grid_1d(n)), dim3(256), 0, s, u, df, n);
  return hipGetLastError();
}

hipError_t launch_bw_add(float* dst, const float* src, int64_t n, hipStream_t s) {
  if (n < 1) return hipSuccess;
  hipLaunchKernelGGL(add_kernel, dim3(grid_1d(n)), dim3(256), 0, s, dst, src, n);
  return hipGetLastError();
}

hipError_t launch_bw_attention(int dtype, const void* qkv, const float* dctx, const int32_t* lengths, int batch, int seq, int d, int n_head, int causal,
                               float* P, float* dS, float* dqkv, hipStream_t s) {
  if (batch < 1 || seq < 1 || n_head < 1 || seq > kBackwardMaxSeq || d % n_head != 0) return hipErrorInvalidValue;
  const int dh = d / n_head, heads = batch * n_head;
  // head z = (b, h): the [T, T] buffers are consecutive in z; q, k, v of the head are the columns h dh, d + h dh, 2 d + h dh of
  // the [T, 3 d] rows of sequence b, dctx its columns h dh of [T, d] rows
  const int64_t tt = (int64_t)seq * seq, ld = (int64_t)3 * d;
  const float scale = 1.0f / sqrtf((float)dh);
  const int64_t sq_outer = (int64_t)seq * ld, dc_outer = (int64_t)seq * d, p_outer = n_head * tt;
  hipError_t e;
  // S [i][j] = sum_t q[i][t] k[j][t] / sqrt dh
  const BatchOffsets bs{n_head, sq_outer, dh, sq_outer, dh, p_outer, tt};
  if (dtype == 1) e = launch_bw_gemm_batched(reinterpret_cast<const bf16_t*>(qkv), ld, 1, dtype, reinterpret_cast<const bf16_t*>(qkv) + d, 1, ld, P, seq, seq, seq, dh, scale, 0, heads, bs, s);
  else            e = launch_bw_gemm_batched(reinterpret_cast<const float*>(qkv), ld, 1, dtype, reinterpret_cast<const float*>(qkv) + d, 1, ld, P, seq, seq, seq, dh, scale, 0, heads, bs, s);
  if (e != hipSuccess) return e;
  // dP [i][j] = sum_t dctx[i][t] v[j][t]
  const void* v0 = dtype == 1 ? (const void*)(reinterpret_cast<const bf16_t*>(qkv) + 2 * d) : (const void*)(reinterpret_cast<const float*>(qkv) + 2 * d);
  e = launch_bw_gemm_batched(dctx, (int64_t)d, 1, dtype, v0, 1, ld, dS, seq, seq, seq, dh, 1.0f, 0, heads, BatchOffsets{n_head, dc_outer, dh, sq_outer, dh, p_outer, tt}, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_backward_rows_kernel, dim3((unsigned)heads * seq), dim3(256), 0, s, lengths, seq, n_head, causal, P, dS);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  // dQ [i][t] = sum_j dS[i][j] k[j][t] / sqrt dh
  const void* k0 = dtype == 1 ? (const void*)(reinterpret_cast<const bf16_t*>(qkv) + d) : (const void*)(reinterpret_cast<const float*>(qkv) + d);
  e = launch_bw_gemm_batched(dS, (int64_t)seq, 1, dtype, k0, ld, 1, dqkv, ld, seq, dh, seq, scale, 0, heads, BatchOffsets{n_head, p_outer, tt, sq_outer, dh, sq_outer, dh}, s);
  if (e != hipSuccess) return e;
  // dK [j][t] = sum_i dS[i][j] q[i][t] / sqrt dh,  dV [j][t] = sum_i P[i][j] dctx[i][t]
  e = launch_bw_gemm_batched(dS, 1, (int64_t)seq, dtype, qkv, ld, 1, dqkv + d, ld, seq, dh, seq, scale, 0, heads, BatchOffsets{n_head, p_outer, tt, sq_outer, dh, sq_outer, dh}, s);
  if (e != hipSuccess) return e;
  return launch_bw_gemm_batched(P, 1, (int64_t)seq, 0, dctx, (int64_t)d, 1, dqkv + 2 * d, ld, seq, dh, seq, 1.0f, 0, heads, BatchOffsets{n_head, p_outer, tt, dc_outer, dh, sq_outer, dh}, s);
}

hipError_t launch_bw_embedding(const int32_t* tok, const float* dx, int M, int seq, int d, int vocab, float* dE, float* dPe, int max_pos, hipStream_t s) {
  hipLaunchKernelGGL(embed_backward_kernel, dim3((unsigned)((d + 255) / 256)), dim3(256), 0, s, tok, dx, M, seq, d, vocab, dE, dPe, max_pos);
  return hipGetLastError();
}

}  // namespace zgr
