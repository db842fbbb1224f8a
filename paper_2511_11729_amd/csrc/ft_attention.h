// Fused causal self-attention of the finetune unit (forward and backward), head_dim 64 or 128.
// Tensors are token-major 16-bit (the compute element of ft_elem.h): q, o, dO, dq, dkq, dvq are [Bf*S, n_q*d];
// k, v are [Bf*S, n_kv*d]; the "T" operands are per-sequence transposes [Bf][heads*d][S].  lse and delta are
// fp32 [Bf*n_q][S].  S must be a multiple of 8.  Query head j reads KV head j / (n_q / n_kv).
#pragma once
#include <hip/hip_runtime.h>

#include "common.h"

namespace harli {
typedef unsigned short bf;

inline bool ft_attn_supported(int d) { return d == 64 || d == 128; }

// o = softmax(q k^T / sqrt(d), causal) v ;  lse[z][s] = log sum_k exp(score[s][k])   (natural log)
harli_status ft_attn_fwd(const bf* q, const bf* k, const bf* vT, bf* o, float* lse, int Bf, int S, int n_q, int n_kv, int d,
                         hipStream_t st);

// Given dO and the forward output o:  delta[z][s] = sum_e dO[s][e] o[s][e] (written to `delta`, a workspace of
// Bf*n_q*S floats),
//   dq  = dS k / sqrt(d),  dkq = dS^T q / sqrt(d),  dvq = P^T dO   with P = exp(score - lse), dS = P (dP - delta),
//   dP = dO v^T.  dkq and dvq are per QUERY head ([Bf*S, n_q*d]); the caller sums them over the heads of a group.
harli_status ft_attn_bwd(const bf* q, const bf* k, const bf* v, const bf* o, const bf* qT, const bf* kT, const bf* dO,
                         const bf* dOT, const float* lse, float* delta, bf* dq, bf* dkq, bf* dvq, int Bf, int S, int n_q,
                         int n_kv, int d, int* flag, hipStream_t st);
}  // namespace harli
