// Internal definition of the model context.
#pragma once
#include <hip/hip_runtime.h>

#include <unordered_map>
#include <vector>

#include "common.h"

#define HARLI_HIP(call)                                                                      \
  do {                                                                                       \
    hipError_t e_ = (call);                                                                  \
    if (e_ != hipSuccess)                                                                    \
      return harli::fail(HARLI_ERR_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)

namespace harli {

constexpr int kTargets = 7;  // q,k,v,o,gate,up,down

struct LayerDev {
  const void* w[kTargets];   // wq wk wv wo wg wu wd, [out,in]
  void* wt[kTargets];        // library-owned transposes [in,out] for the backward pass (after lora_attach)
  void* w16[kTargets];       // library-owned [out,in] copies in the finetune compute element (after lora_attach)
  void* wp[kTargets];        // decode-private pre-shuffled copies: [0] = q,k,v stacked, [3] o, [4] gate, [5] up, [6] down
  const float *g1, *g2;
  const float* bias[3];      // borrowed q, k, v biases (fp32) or null
  void* b16[3];              // library-owned [out, 8] copies in the finetune compute element, bias in column 0 (after lora_attach)
  void* A[kTargets];         // borrowed adapter pointers (NULL when not adapted)
  void* B[kTargets];
};

// Device buffers of the decode path, sized by max_batch (rounded up to 16).
struct DecodeWs {
  int bpad = 0;
  void *hx1 = nullptr, *obuf = nullptr, *hx2 = nullptr, *mbuf = nullptr;  // GEMM operands in storage dtype
  float *qbuf = nullptr, *x1 = nullptr, *xa = nullptr, *xb = nullptr;    // fp32
  float* ssq = nullptr;       // [2*L+1][bpad][ssq_entries(hidden)]: per-tile partial sums of squares of the residual rows
  float* rope = nullptr;      // [bpad][d/2][2]
  double* inv_freq = nullptr; // [d/2] base^(-2i/d)
  float* att_part = nullptr;  // [bpad][n_q][max_chunks][d+2]
  float* amax_v = nullptr;    // [bpad][64] per-slice maxima of the logits (full-model mode)
  int* amax_i = nullptr;      // [bpad][64] and their indices
  float* scores = nullptr;    // fp32 path only: [bpad][n_q][max_seq_len]
  float *fk = nullptr, *fv = nullptr, *fa = nullptr, *fu = nullptr;  // fp32 path only: k, v [bpad, n_kv*d]; gate, up [bpad, ffn]
  int* err_flag = nullptr;    // device int set when a kernel sees an out-of-range page id
  int max_chunks = 0;
  float* part = nullptr;      // partial tiles of the large-batch GEMMs (null: batches stay on the small-batch kernels)
  size_t part_bytes = 0;
};

}  // namespace harli

struct harli_ctx {
  harli_model_cfg cfg{};
  harli_pool* pool = nullptr;
  harli::KvGeom geom{};
  char* slab = nullptr;
  std::vector<harli::LayerDev> layers;
  const void* emb = nullptr;
  const float* g_final = nullptr;
  const void* w_lm = nullptr;
  void* wlm_p = nullptr;     // pre-shuffled output layer
  harli::DecodeWs dw;
  // LoRA / finetune state
  bool lora_attached = false;
  harli_lora_cfg lora{};
  void* ft_ws = nullptr;     // finetune workspace (library-owned)
  size_t ft_ws_bytes = 0;
  void* head_ws = nullptr;   // output-layer workspace of the finetune task (library-owned)
  void* ones16 = nullptr;    // [max_ft_tokens, 8] ones in the finetune compute element: the input column of the biases
  void* window = nullptr;    // window over the finetune task's frozen weights (library-owned), or null
  int n_cu = 0;
  size_t decode_ws_bytes = 0, decode_weight_bytes = 0;  // device memory harli_ctx_create allocated
  std::unordered_map<void*, harli_alloc> pool_allocs;   // library buffers that are allocations of the pool (cfg.memory_in_pool)
};

namespace harli {
// entries per row of DecodeWs::ssq: one per 16 columns of the hidden size, padded to a multiple of 16
inline int ssq_entries(int hidden) { return (((hidden + 15) >> 4) + 15) & ~15; }
// A device buffer the library keeps for the context: from the pool when cfg.memory_in_pool is set (HARLI_ERR_OOM when
// it has no room), else a library allocation.  lib_free takes either kind (and null).
harli_status lib_alloc(harli_ctx* c, void** p, size_t bytes);
void lib_free(harli_ctx* c, void* p);
size_t packed_weight_elems(int N, int K);
harli_status pack_weight(const void* src, void* dst, int N, int K, int row_tile0, hipStream_t st);
// element size of the storage dtype
inline size_t esize(const harli_ctx* c) { return c->cfg.dtype == HARLI_BF16 ? 2 : 4; }
inline void proj_shape(const harli_model_cfg& m, int t, int* out, int* in) {
  int q = m.n_q_heads * m.head_dim, kv = m.n_kv_heads * m.head_dim;
  switch (t) {
    case 0: *out = q; *in = m.hidden; break;
    case 1: case 2: *out = kv; *in = m.hidden; break;
    case 3: *out = m.hidden; *in = q; break;
    case 4: case 5: *out = m.ffn; *in = m.hidden; break;
    default: *out = m.hidden; *in = m.ffn; break;
  }
}
}  // namespace harli
