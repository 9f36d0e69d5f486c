// Host-callable launchers of the backward-pass kernels (backward.hip): the cloud block of Algorithm 1.
// dtype / b_dtype: 0 = fp32 storage, 1 = bf16 storage.  All pointers are device memory; gradients are fp32.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zgr {

constexpr int kBackwardMaxSeq = 2048;      // keys one workgroup of the attention rule holds

// C[i][j] (+)= alpha sum_k A[i ars + k acs] B[k brs + j bcs]; A fp32, B of b_dtype
hipError_t launch_bw_gemm(int b_dtype, const float* A, int64_t ars, int64_t acs, const void* B, int64_t brs, int64_t bcs, float* C, int64_t ldc,
                          int M, int N, int K, float alpha, int accumulate, hipStream_t s);
// bf16 operands for the matrix-core products: out [cols, rows] (row stride ld_out) = in [rows, cols]^T, in fp32 or bf16
// (row stride ld_in); out [rows, cols] (row stride ld_out) = in rounded.  What lies between the data and ld_out is written as zeros.
hipError_t launch_bw_transpose_bf16(int in_dtype, const void* in, int rows, int cols, int64_t ld_in, void* out, int64_t ld_out, hipStream_t s);
hipError_t launch_bw_round_bf16(const float* in, int rows, int cols, int64_t ld_in, void* out, int64_t ld_out, hipStream_t s);
// out[n] = sum_m Y[m ld + n]; part: scratch of bw_colsum_scratch_floats(N) floats
size_t     bw_colsum_scratch_floats(int n_max);
hipError_t launch_bw_colsum(const float* Y, int M, int N, int64_t ld, float* out, float* part, hipStream_t s);
hipError_t launch_bw_fill(float* p, int64_t n, float v, hipStream_t s);
// logits [rows, n] -> (softmax - onehot(target)) inv_count in place; rows with a target outside [0, n) become zeros
hipError_t launch_bw_cross_entropy(float* logits, const int32_t* targets, int rows, int n, float inv_count, hipStream_t s);
// y = LayerNorm(x) g + b: dx_out = (add ? add : 0) + dL/dx (dx_out may be add or dy), dg, db from dy; stats: 2 M floats of scratch, part: bw_colsum_scratch_floats(d)
hipError_t launch_bw_layernorm(int dtype, const float* x, const void* g, const float* dy, const float* add, float* dx_out, float* stats, float* dg, float* db,
                               float* part, int M, int d, float eps, hipStream_t s);
// f = act(u) in the storage type (erf-GELU, or ReLU when relu != 0); df <- df act'(u); dst += src
hipError_t launch_bw_act_forward(int dtype, int relu, const float* u, void* f, int64_t n, hipStream_t s);
hipError_t launch_bw_act(int relu, const float* u, float* df, int64_t n, hipStream_t s);
hipError_t launch_bw_add(float* dst, const float* src, int64_t n, hipStream_t s);
// dqkv [B T, 3 d] from dctx [B T, d]; P, dS: scratch of B n_head T T floats each
hipError_t launch_bw_attention(int dtype, const void* qkv, const float* dctx, const int32_t* lengths, int batch, int seq, int d, int n_head, int causal,
                               float* P, float* dS, float* dqkv, hipStream_t s);
// dE [vocab, d] += rows of dx by token, dPe [max_pos, d] = sums of dx by position
hipError_t launch_bw_embedding(const int32_t* tok, const float* dx, int M, int seq, int d, int vocab, float* dE, float* dPe, int max_pos, hipStream_t s);

}  // namespace zgr
