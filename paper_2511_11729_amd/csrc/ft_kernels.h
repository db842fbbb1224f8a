// Element-wise, reduction and skinny kernels of the finetune unit (launch wrappers).
// All tensors are device pointers; "bf" = one 16-bit element (the compute element of ft_elem.h unless a
// name says bf16), rows are token-major.
#pragma once
#include <hip/hip_runtime.h>

#include "common.h"

namespace harli {
typedef unsigned short bf;

// h = bf16(x * rho * g), rho = rsqrt(mean x^2 + eps) (also stored)
void ft_rmsnorm_fwd(const float* x, const float* g, bf* h, float* rho, int T, int H, float eps, int* flag, hipStream_t st);
// dx = dres + rho * (dh*g - xhat * mean(dh*g*xhat)), xhat = x*rho;  dh is fp32
// res_mul / out_mul: optional device scalars: dx = out_mul * (dres * res_mul + ...); dres may be NULL (taken as zero)
// dx16: optional 16-bit copy of dx (the next GEMM's operand)
void ft_rmsnorm_bwd(const float* dh, const float* x, const float* rho, const float* g, const float* dres, float* dx, bf* dx16,
                    int T, int H, const float* res_mul, const float* out_mul, int* flag, hipStream_t st);
// rotary embedding in place on [T, heads*d] bf16, position = t % S; inverse rotates by the negative angle
void ft_rope(bf* t, int T, int S, int heads, int d, const double* inv_freq, bool inverse, int* flag, hipStream_t st);
// Gradient scaling in two launches: the largest |x| (n a multiple of 4), then y = 16-bit(x * sigma) with sigma the power
// of two that brings it to 2^target_log2; scale[0] = sigma and scale[1] = 1 / sigma are left for the kernels downstream.
// scale[2], scale[3] hold the maximum (as bits) of this call and the next: they must be zero before the first call, and
// `parity` alternates between calls (each call clears the slot of the next).
void ft_scale_to_e(const float* x, bf* y, long long n, float* scale, int parity, int target_log2, hipStream_t st);
// Several storage -> compute-element conversions in one launch: src [R][C] (bf16, or fp32 when src_f32 is set) ->
// dst [R][C], or dst [C][R] when transpose is set (meant for adapter matrices and one-time weight copies: the
// strided side is not tuned)
struct FtConvJob {
  const void* src;
  bf* dst;
  int R, C, transpose, src_f32;
};
struct FtConvJobs {
  FtConvJob j[16];
  int n;
  int* flag;  // device int or null: bit 8 is set when a value lay beyond the compute element's range
};
void ft_convert_jobs(const FtConvJobs& jobs, hipStream_t st);
// head-wise transposes of [Bf*S, C] tensors (C = heads * d, S and C multiples of 8) into [Bf][C][S], up to three in one
// launch
struct TransposeJobs {
  const bf* in[3];
  bf* out[3];
  int C[3];
  int n;
};
void ft_transpose_heads(const TransposeJobs& jobs, int Bf, int S, hipStream_t st);
// skinny NT GEMMs: C[M, N] = alpha * X[M, K] . Bm[N, K]^T, N <= 64 and N % 16 == 0 after padding by the caller's layout;
// several such products with the same M and alpha in one launch (job = blockIdx.y).
constexpr int kSkinnyMaxJobs = 4;
struct SkinnyNtJob {
  const bf* X;
  long long ldx;
  const bf* Bm;
  long long ldb;
  bf* C;
  long long ldc;
  int N, K;
};
struct SkinnyNtJobs {
  int n;
  SkinnyNtJob j[kSkinnyMaxJobs];
};
void ft_skinny_nt_multi(const SkinnyNtJobs& jobs, int M, float alpha, int* flag, hipStream_t st);
// G[j*sj + r*sr] += out_mul * sum_t X[t][j] * U[t][r];  X [T, J] and U [T, R] 16-bit, R in {8, 16, 32, 64}, J even,
// one of sj, sr equal to 1.  `part` is scratch of ft_lora_grad_ws_floats(J, R) floats; G is read and written
// without atomics, so no other work may update it concurrently.
size_t ft_lora_grad_ws_floats(int J, int R);
// Several such products in one pair of launches (their workgroups run side by side instead of one short kernel after
// the other): job i is G_i[j*sj + r*sr] += out_mul * sum_t X_i[t][j] * U_i[t][r] with its own J; same T and R for all.
// The host fills X, ldx, U, ldu, G, sj, sr, J; the remaining fields are set by ft_lora_grad_multi.
constexpr int kLoraGradMaxJobs = 8;
struct LoraGradJob {
  const bf* X;
  long long ldx;
  const bf* U;
  long long ldu;
  float* G;
  long long sj, sr;
  int J;
  int jt, nch, tpm;    // column tiles, token chunks, tokens per chunk
  long long part_off;  // this job's partial sums inside the scratch
};
struct LoraGradJobs {
  int n;
  LoraGradJob j[kLoraGradMaxJobs];
};
void ft_lora_grad_multi(LoraGradJobs& jobs, int T, int R, const float* out_mul, float* part, hipStream_t st);
void ft_lora_grad(const bf* X, long long ldx, const bf* U, long long ldu, float* G, long long sj, long long sr, int T, int J,
                  int R, const float* out_mul, float* part, hipStream_t st);
// sum GQA query-head groups: dk[T][n_kv*d] = sum_g dkq[T][(c*G+g)*d + e]
void ft_sum_groups(const bf* in, bf* out, int T, int n_kv, int G, int d, int* flag, hipStream_t st);
}  // namespace harli
