// Host-callable launchers of the forward-pass kernels (forward.hip).
// dtype: 0 = fp32 storage, 1 = bf16 storage.  All pointers are device memory.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zgr {

enum { EPI_STORE = 0, EPI_GELU = 1, EPI_RESID = 2, EPI_F32 = 3, EPI_CE = 4, EPI_RELU = 5 };

hipError_t launch_embed(int dtype, const int32_t* tok, const void* E, const void* Pe, float* x, int M, int seq, int d, int vocab, hipStream_t s);
// out (storage type) = LayerNorm(x) g + b; xout, when not NULL, receives the same values in fp32 (it may be x itself)
hipError_t launch_layernorm(int dtype, const float* x, const void* g, const void* b, void* out, int M, int d, float eps, hipStream_t s, float* xout = nullptr);
// out = epilogue(A[M,K] W[N,K]^T + bias); bf16 storage needs K % 64 == 0.
hipError_t launch_gemm(int dtype, const void* A, const void* W, const void* bias, void* out, int epi, int M, int N, int K, hipStream_t s);
// bf16 vocabulary projection fused with cross-entropy: row_loss[m] = logsumexp(A[m] W^T) - (A[m] W^T)[targets[m]] (0 where targets[m] < 0).
int        ce_partials_per_row(int N);
hipError_t launch_gemm_ce_bf16(const void* A, const void* W, const int32_t* targets, void* part, float* tlogit, float* row_loss, int M, int N, int K, hipStream_t s);
hipError_t launch_attention(int dtype, const void* qkv, void* ctx, const int32_t* lengths, int batch, int seq, int d, int n_head, int causal, hipStream_t s);
bool       attention_head_dim_supported(int dh);
hipError_t launch_lm_targets(const int32_t* tok, int32_t* tgt, int M, int seq, int vocab, hipStream_t s);
hipError_t launch_ce_rows(const float* logits, const int32_t* targets, float* row_loss, int M, int n, hipStream_t s);
hipError_t launch_mean_f64(const float* v, int n, double inv_count, double* out, hipStream_t s);
hipError_t launch_cls_head(int dtype, const void* h, const void* Wc, const void* bc, float* logits, int batch, int seq, int d, int n_class, hipStream_t s);
hipError_t launch_lsq_rows(const float* pred, const float* Y, float* row_loss, int batch, int n_out, hipStream_t s);

}  // namespace zgr
