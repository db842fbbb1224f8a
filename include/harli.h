/*
 * harli.h -- C ABI of the MI355X (gfx950) hot path of Harli (arXiv 2511.11729):
 * a memory-bound small-batch LLM decode step co-located on one GPU with a
 * compute-bound LoRA finetune step, both drawing memory from one unified pool.
 *
 * General rules
 *  - Every call returns a harli_status; nothing throws or aborts across the ABI;
 *    out-parameters are written only on HARLI_OK.  harli_last_error() returns a
 *    thread-local, human-readable description of the last failure.
 *  - "device" pointers are HIP device addresses, "host" pointers ordinary memory.
 *  - The caller owns the slab, all weights, adapters, input/output buffers and
 *    both streams.  The library owns host bookkeeping, the per-context device
 *    workspace it allocates in harli_ctx_create / harli_lora_attach, and the
 *    harli_saved records (whose device bytes live inside the caller's slab).
 *  - Compute calls are asynchronous on the stream they are given and never
 *    synchronise the device.  A context may run harli_decode_step on one stream
 *    and harli_lora_fwd/bwd on another concurrently (Sec. 7: two model instances
 *    in one process, each on its own stream); two decode steps, or two finetune
 *    calls, of the same context must not overlap.
 *  - Storage type: HARLI_BF16 (weights, KV cache and saved activations are
 *    bfloat16, accumulation is fp32) or HARLI_F32 (weights, adapters and KV cache are
 *    fp32; decode computes in fp32 throughout, the finetune unit rounds weights and
 *    adapters to its 16-bit compute element and keeps fp32 accumulation).  Hidden
 *    states crossing the ABI (x, y, dY, dX), RMSNorm gains, logits and adapter
 *    gradients are always fp32.
 *  - Linear weights are [out, in] row-major (y = x W^T), no biases.  LoRA A is
 *    [in, r], B is [r, out], y = x W^T + (alpha/r) (x A) B.
 *  - Rotary embedding pairs element i with i + head_dim/2.
 */
#ifndef HARLI_H
#define HARLI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HARLI_OK = 0,
  HARLI_ERR_INVALID = 1, /* bad argument or unsupported shape */
  HARLI_ERR_OOM = 2,     /* the pool (or the device) cannot serve the request */
  HARLI_ERR_STATE = 3,   /* call not valid in the object's current state */
  HARLI_ERR_HIP = 4      /* a HIP runtime call failed */
} harli_status;

typedef enum { HARLI_BF16 = 0, HARLI_F32 = 1 } harli_dtype;

const char* harli_status_str(harli_status s);
const char* harli_last_error(void);
/* Library version string (static storage). */
const char* harli_version(void);

/* ======================================================================== *
 * Unified memory pool (Sec. 4.2, 4.4, 4.5).  Host-side bookkeeping over ONE
 * caller-owned device slab; no call here touches device memory.
 *
 * Slab layout:  [ small-tensor pool | chunk 0 | chunk 1 | ... ]
 *   chunk  = n_layers x 2 blocks (Sec. 4.2); FREE, KV or TENSOR; returns to
 *            FREE when everything in it is released.
 *   block  = block_bytes (2 MiB in the paper).  In a KV chunk, block
 *            2*layer + kv holds that layer's K (kv=0) or V (kv=1).
 *   page   = page_tokens (16) consecutive tokens; pages_per_block =
 *            floor(block_bytes / (page_tokens * kv_row_bytes)).  A page id is
 *            chunk * pages_per_block + slot and names the same token run in
 *            every layer's K and V -- one column of the paper's 2-D grid.
 *            Inside a page the element order is [kv head][token slot][head_dim]
 *            (the paper fixes the grid, not the order inside an entry; head-major
 *            keeps one head's 16 tokens contiguous for the attention kernel).
 *   small  = buddy allocator, granule small_granule (2 KiB, Sec. 4.5), made of
 *            arenas of block_bytes each.
 * Placement policy is "lowest index first" everywhere, so ids and offsets are
 * reproducible.  KV pages may take any FREE chunk; tensor allocations must
 * leave kv_reserve_chunks FREE chunks behind (inference priority, Sec. 4.4)
 * and get HARLI_ERR_OOM otherwise.
 * All pool calls are thread-safe (one mutex) and O(chunks) at worst.
 * ======================================================================== */
typedef struct harli_pool harli_pool;

typedef struct {
  size_t block_bytes;       /* power-of-two multiple of small_granule; paper: 2 MiB */
  int32_t n_layers;         /* layerNum of the inference model */
  int32_t page_tokens;      /* tokens per KV page (16) */
  size_t kv_row_bytes;      /* n_kv_heads * head_dim * element size */
  size_t small_pool_bytes;  /* multiple of block_bytes (may be 0) */
  size_t small_granule;     /* paper: 2 KiB */
  int32_t kv_reserve_chunks;
} harli_pool_cfg;

typedef enum { HARLI_CLS_KV_PAGE = 0, HARLI_CLS_TENSOR = 1, HARLI_CLS_SMALL = 2, HARLI_CLS_AUTO = 3 } harli_class;

typedef struct {
  int32_t cls;      /* class that served the request (SMALL may fall back to TENSOR) */
  int32_t page;     /* KV_PAGE: page id; otherwise -1 */
  size_t offset;    /* TENSOR / SMALL: byte offset from the slab base */
  size_t bytes;     /* bytes reserved (request rounded up to blocks / buddy order) */
  void* ptr;        /* slab + offset (device); NULL for KV_PAGE */
} harli_alloc;

typedef struct {
  int32_t n_chunks, free_chunks, kv_chunks, tensor_chunks;
  int32_t pages_per_block, blocks_per_chunk;
  int64_t kv_pages_live, tensor_blocks_live;
  size_t small_bytes_live;     /* reserved bytes in the buddy pool */
  size_t requested_bytes_live; /* sum of requested sizes of live TENSOR/SMALL allocations */
  size_t reserved_bytes_live;  /* sum of reserved sizes of the same allocations */
  int64_t small_fallbacks;     /* SMALL requests served by a TENSOR block */
  int64_t pending_frees;       /* frees still waiting for their event */
} harli_pool_stats_t;

/* slab: device base address (never dereferenced); slab_bytes >= small_pool_bytes + one chunk. */
harli_status harli_pool_create(void* slab, size_t slab_bytes, const harli_pool_cfg* cfg, harli_pool** out);
/* Gives up the creator's hold on the pool.  A context built on the pool (harli_ctx_create) holds it too and returns its
 * pool memory when it is destroyed: the pool object is deleted when the last holder is gone, so the two may be destroyed
 * in either order.  The caller must not use p after this call. */
void harli_pool_destroy(harli_pool* p);

/* One allocation.  cls = KV_PAGE: n is ignored, one page is returned in out->page.
 * TENSOR: n bytes, rounded up to whole blocks, contiguous.  SMALL: n < block_bytes,
 * rounded up to small_granule * 2^k.  AUTO: SMALL if n < block_bytes else TENSOR. */
harli_status harli_pool_alloc(harli_pool* p, harli_class cls, size_t n, harli_alloc* out);
/* n_pages KV pages at once into page_ids (host).  All or nothing. */
harli_status harli_pool_alloc_pages(harli_pool* p, int32_t n_pages, int32_t* page_ids);

/* Release.  `event` is a hipEvent_t (or NULL): when given, the memory becomes
 * reusable only once hipEventQuery(event) reports completion (polled on later
 * pool calls); the caller keeps the event alive until then.  Double free or an
 * unknown allocation is HARLI_ERR_INVALID. */
harli_status harli_pool_free(harli_pool* p, const harli_alloc* a, void* event);
harli_status harli_pool_free_pages(harli_pool* p, int32_t n_pages, const int32_t* page_ids, void* event);

/* Byte offset from the slab base of page `page` of layer `layer`'s K (kv=0) or V (kv=1):
 * small_pool_bytes + chunk*chunk_bytes + (2*layer+kv)*block_bytes + slot*page_bytes. */
harli_status harli_pool_kv_addr(const harli_pool* p, int32_t page, int32_t layer, int32_t kv, size_t* byte_off);
harli_status harli_pool_stats(harli_pool* p, harli_pool_stats_t* out);

/* Inter-task memory coordination (Sec. 4.4, Principle 3).
 * reserve_chunks_for: the number of chunks that hold Memory_reserved = (T / SLO) * max_bs * Mem_kv at page
 *   granularity, where release_time (T) is how long the finetune task needs to give memory back and slo the decode
 *   QoS target (same unit) and max_bs the largest decode batch: in ceil(T / SLO) decode steps each sequence appends
 *   that many tokens and may need ceil(steps / page_tokens) new pages, so the reserve is
 *   ceil(max_bs * ceil(ceil(T / SLO) / page_tokens) / pages_per_block) chunks.  Pure arithmetic on the geometry.
 * set_reserve: replaces kv_reserve_chunks (it only gates FUTURE tensor-chunk conversions; nothing is evicted).
 * pressure: how many chunks the finetune task should relinquish now = min(max(0, reserve - FREE chunks),
 *   TENSOR chunks); polls pending event-deferred frees first.  The caller answers by releasing saved
 *   activations / skipping finetune units until it reads 0. */
harli_status harli_pool_reserve_chunks_for(const harli_pool* p, double release_time, double slo, int32_t max_bs, int32_t* chunks);
harli_status harli_pool_set_reserve(harli_pool* p, int32_t chunks);
harli_status harli_pool_pressure(harli_pool* p, int32_t* chunks_to_release);

/* ======================================================================== *
 * Model context: shapes plus BORROWED device pointers to the frozen weights.
 * ======================================================================== */
typedef struct harli_ctx harli_ctx;

typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  float rms_eps;    /* 1e-6 */
  float rope_base;  /* 10000 */
  int32_t dtype;    /* harli_dtype: storage of weights, KV cache, saved activations */
  int32_t max_batch;      /* largest decode batch (1..256).  From 17 on the context also holds the workspace of the tiled
                           * GEMMs that steps of more than 32 sequences run (Sec. 1: decode is served up to batch 256):
                           * up to 192 MiB for the partial tiles, part of decode_workspace in harli_ctx_device_bytes */
  int32_t max_seq_len;    /* largest kv_len[b] + 1 a decode step may see */
  int32_t max_ft_tokens;  /* largest B_f*S of a finetune call (0: finetune unused) */
  /* Where the library's own device memory for this context lives: the decode instance's pre-shuffled weight copies and
   * step buffers, the finetune instance's weight copies, and both workspaces.  0: the library allocates it.  1: all of
   * it is taken from the unified pool (Sec. 4.2: one pool holds every tensor of both tasks; TENSOR allocations, small
   * buffers from the SMALL pool), so that harli_pool_stats accounts for every byte the context holds, and
   * harli_ctx_create / harli_lora_attach return HARLI_ERR_OOM when the pool cannot hold it (the caller sizes the slab:
   * harli_ctx_device_bytes reports what a context took).  It implies harli_lora_cfg.workspace_in_pool. */
  int32_t memory_in_pool;
} harli_model_cfg;

typedef struct {
  const void *wq, *wk, *wv, *wo, *wg, *wu, *wd; /* device, [out,in], cfg.dtype */
  const float *g1, *g2;                         /* device, [hidden] RMSNorm gains */
  const float *bq, *bk, *bv; /* device fp32 [n_q*head_dim], [n_kv*head_dim], [n_kv*head_dim]: frozen biases added to the
                              * q, k, v projections before the rotary embedding (the Qwen2.5 family, Sec. 8.1), or NULL */
} harli_layer_weights;

typedef struct {
  const harli_layer_weights* layers; /* host array of n_layers entries (copied) */
  const void* emb;                   /* device [vocab, hidden] or NULL */
  const float* g_final;              /* device [hidden] or NULL */
  const void* w_lm;                  /* device [vocab, hidden] or NULL */
} harli_weights;

/* The pool supplies the KV cache geometry and the slab; it must outlive the context.
 * Allocates a device workspace proportional to max_batch and max_ft_tokens. */
harli_status harli_ctx_create(const harli_model_cfg* cfg, const harli_weights* w, harli_pool* pool, harli_ctx** out);
void harli_ctx_destroy(harli_ctx* c);
/* Device memory the context holds beyond the caller's buffers (host out-pointer; host arithmetic only).  The decode
 * instance keeps a private, pre-shuffled copy of the frozen weights and a small workspace (both made by
 * harli_ctx_create); the finetune instance keeps private copies W and W^T of the frozen weights in its compute element
 * (made by harli_lora_attach; the paper also keeps one model instance per task, Sec. 7) and the workspace described at
 * harli_lora_cfg.  `in_pool` of these bytes are allocations of the unified pool, `outside_pool` are the library's own.
 * After harli_ctx_create and harli_lora_attach the library no longer reads the seven projection matrices of a layer
 * or w_lm on bf16 storage (everything runs on its copies): a caller short of memory may free them.  emb, the norm
 * gains, biases and the adapters stay borrowed. */
typedef struct {
  size_t decode_weights, decode_workspace;
  size_t finetune_weights, finetune_workspace;
  size_t head_weights, head_workspace;
  size_t in_pool, outside_pool;
} harli_device_bytes;
harli_status harli_ctx_device_bytes(const harli_ctx* c, harli_device_bytes* out);

/* Diagnostic, SYNCHRONISES `hip_stream`: reports (and clears) whether any kernel of this
 * context met a page id outside the pool or a token id outside the vocabulary.  Such
 * entries are skipped by the kernels, never dereferenced. */
harli_status harli_ctx_check(harli_ctx* c, void* hip_stream);

/* ---- LoRA adapters (Sec. 2.1: only the adapters are trainable) -------------- */
enum { HARLI_T_Q = 1, HARLI_T_K = 2, HARLI_T_V = 4, HARLI_T_O = 8, HARLI_T_GATE = 16, HARLI_T_UP = 32, HARLI_T_DOWN = 64 };

typedef struct {
  int32_t rank;
  float alpha;       /* scale = alpha / rank */
  uint32_t targets;  /* bit mask of HARLI_T_* */
  /* Where the finetune task's workspace lives (backward temporaries of one unit and the output layer's logits chunk,
   * sized once for max_ft_tokens in harli_lora_attach; no forward / backward call allocates afterwards).  0: the
   * library allocates it.  1: it is taken from the unified pool as TENSOR allocations (Sec. 4.2: one pool for every
   * tensor of both tasks), so harli_pool_stats and the inference-first coordination of Sec. 4.4 account for it; the
   * caller sizes the slab for it (harli_ctx_device_bytes reports the size) and harli_lora_attach returns
   * HARLI_ERR_OOM when the pool cannot hold it. */
  int32_t workspace_in_pool;
  /* The backward pass carries gradients in IEEE half, scaled by the power of two that brings max|dY| of the unit to
   * 2^(8 - grad_headroom_log2): the default 0 keeps small gradients well above half's underflow; a model whose
   * activations have outlier channels (gradients of the gated FFN are products with them) can overflow half at that
   * scale, which harli_ctx_check reports; such a caller gives headroom here (0..24).  The results are unscaled
   * before they are returned; the scale itself changes no bit of them while nothing under- or overflows. */
  int32_t grad_headroom_log2;
} harli_lora_cfg;

/* A, B: host arrays of n_layers*7 device pointers indexed [layer*7 + t], t = 0..6
 * for q,k,v,o,gate,up,down (entries of non-adapted projections are ignored);
 * rank must be 8, 16, 32 or 64.
 * Borrowed; the caller may update their contents between calls (optimizer step).
 * Also builds library-owned transposed copies of the frozen weights that the
 * backward pass streams (dx = dy W needs W with `in` as the slow axis). */
harli_status harli_lora_attach(harli_ctx* c, const harli_lora_cfg* cfg, void* const* A, void* const* B);

/* ======================================================================== *
 * Decode step (Sec. 2.1: one new token per sequence; Sec. 4.1: KV slots by index).
 * For every layer: RMSNorm, Q/K/V projection, rotary embedding at position
 * kv_len[b], append K/V to page page_table[b][kv_len[b]/page_tokens] at slot
 * kv_len[b]%page_tokens, attention over positions 0..kv_len[b], output
 * projection + residual, SwiGLU FFN + residual.  Base weights only.
 * ======================================================================== */
typedef struct {
  int32_t batch;              /* 1..cfg.max_batch */
  const int32_t* token_ids;   /* device [batch] (needs emb) or NULL */
  const float* x_in;          /* device [batch, hidden], used when token_ids is NULL */
  float* x_out;               /* device [batch, hidden]: hidden state after the last layer, or NULL */
  float* logits;              /* device [batch, vocab] (needs g_final, w_lm) or NULL */
  int32_t* next_token;        /* device [batch]: argmax of logits, ties to the lowest index, or NULL */
  const int32_t* kv_len;      /* device [batch]: tokens cached BEFORE this step */
  const int32_t* page_table;  /* device [batch, max_pages]: page ids; must already hold the page of position kv_len[b] */
  int32_t max_pages;          /* row stride of page_table */
  int32_t max_kv_len;         /* host-known upper bound of kv_len[b] + 1 (sizes the attention grid) */
} harli_decode_batch;

harli_status harli_decode_step(harli_ctx* c, const harli_decode_batch* b, void* hip_stream);

/* The same step for callers that cannot allocate device memory or rely on memory allocated for them: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments as harli_decode_step and,
 * up to 32 sequences, the same kernels and the same bits, but every intermediate buffer of the step (GEMM operands,
 * q, attention partials, row norms, rotary table, argmax partials) lives in one array of HARLI_STATIC_SCRATCH_BYTES
 * that is part of the library's device image (each GPU the library runs on holds its copy until the process ends)
 * instead of the workspace harli_ctx_create allocated.  Above 32 sequences harli_decode_step runs its GEMMs tiled over
 * ranges of K with partial tiles in that workspace (tens of MB, which the array has no room for): this entry point
 * then keeps the kernels that take the batch in passes of 64 or 128 rows, and agrees with harli_decode_step to
 * rounding, not bit for bit.  The call itself allocates and frees nothing, on the host side of the
 * device or through any library.  bf16 storage only.
 *   - harli_decode_step_static_bytes(c, batch, max_kv_len) is what a step of that batch and length bound needs
 *     (host arithmetic; 0 for bad arguments).  A step that needs more than HARLI_STATIC_SCRATCH_BYTES is refused
 *     with HARLI_ERR_INVALID before anything is enqueued; every other check is harli_decode_step's.
 *   - Every call on a GPU uses that GPU's one array and finds what the last call left in it; the step clears what
 *     must start at zero with a kernel of its own (no memset node, so the call can be captured).  Two calls that
 *     overlap in time on one GPU -- two streams, two contexts, two threads -- race on the array: keep them in
 *     stream order.  harli_decode_step does not touch the array and may run beside it. */
#define HARLI_STATIC_SCRATCH_BYTES (64u << 20)
harli_status harli_decode_step_static(harli_ctx* c, const harli_decode_batch* b, void* hip_stream);
/* Smallest batch whose harli_decode_step runs the tiled GEMMs (33 unless a measurement hook moved it): the step time
 * is linear in the batch size on either side with different slopes, which a latency predictor may want to know
 * (harli_pred_set_batch_split). */
int32_t harli_decode_tiled_min_batch(void);
size_t harli_decode_step_static_bytes(const harli_ctx* c, int32_t batch, int32_t max_kv_len);

/* ======================================================================== *
 * Finetune unit (Sec. 6.1): one transformer layer x one micro-batch.
 * ======================================================================== */
typedef struct harli_saved harli_saved;

/* Y = layer(X) with LoRA on the attached targets, causal attention over each of
 * the B_f sequences of S tokens (positions 0..S-1).  X, Y: device [B_f*S, hidden]
 * fp32.  The activations the backward pass needs are placed in buffers taken
 * from the pool (TENSOR/SMALL classes) and returned in *saved; X itself is
 * borrowed and must stay valid and unchanged until the matching harli_lora_bwd
 * or harli_saved_release.  HARLI_ERR_OOM leaves nothing allocated.  S must be a
 * multiple of 8; the first call of a (B_f, S) shape grows a library-owned
 * device workspace (hipMalloc). */
harli_status harli_lora_fwd(harli_ctx* c, int32_t layer, const float* X, float* Y, int32_t B_f, int32_t S,
                            harli_saved** saved, void* hip_stream);

/* dX = d loss / dX given dY = d loss / dY (device [B_f*S, hidden] fp32).
 * dA, dB: host arrays of 7 device pointers (q,k,v,o,gate,up,down; fp32, shapes
 * of A and B); the adapter gradients are ACCUMULATED into them (read and written
 * without atomics: nothing else may update them while the call runs).  Frozen weights
 * get no gradient.  Consumes `saved`: its pool memory is released with an event
 * recorded on `hip_stream` after the last kernel. */
harli_status harli_lora_bwd(harli_ctx* c, int32_t layer, const float* dY, float* dX, harli_saved* saved,
                            float* const* dA, float* const* dB, void* hip_stream);

/* Drop a saved record without running backward (forward-only unit). */
harli_status harli_saved_release(harli_ctx* c, harli_saved* saved, void* hip_stream);
/* Pool bytes a forward call of (B_f, S) reserves for its saved activations. */
harli_status harli_saved_bytes(const harli_ctx* c, int32_t B_f, int32_t S, size_t* bytes);

/* ---- Window over the finetune task's frozen weights (Sec. 4.3; shrinking under memory pressure: Sec. 4.4) ----
 * After harli_lora_attach the library holds finetune-private copies of every layer's frozen weights (W for the forward
 * pass, W^T for the backward pass).  harli_ft_window_enable moves them to pinned host memory and keeps only n_slots of
 * them on the device, in TENSOR allocations of the unified pool (one slot = one layer's seven matrices in one
 * orientation, one allocation per matrix; n_slots is capped at 2 * n_layers, which is everything).  A training step uses the copies in a fixed
 * cyclic order -- W of layers 0..L-1, then W^T of layers L-1..0 -- and harli_lora_fwd / harli_lora_bwd make their
 * stream wait for the copy they need, then, once the layer is enqueued, refill its slot over a library-owned copy
 * stream with the nearest copy among the next min(n_slots, 4) in that order that is not on the device; when those are
 * all there the layer's own copy stays.  Up to four slots that is the paper's sliding window (the first layer outside
 * the window replaces the layer just computed: 2L copies per step); with more slots the others keep their copies and a
 * step moves (2L - n_slots) * 2L / (2L - 4) copies on average, so the traffic falls as the window grows.
 * A copy requested while absent (another order of calls, a window just resized) is loaded on demand.  Frozen weights
 * never change, so eviction writes nothing back.  Results are bit-identical with and without a window.
 * enable: HARLI_ERR_STATE before lora_attach or when a window exists; HARLI_ERR_OOM when the pool cannot hold n_slots
 *   slots or the host cannot pin the copies (nothing is moved then).  Synchronises the device.
 * resize: grows (pool permitting: on HARLI_ERR_OOM the window keeps the slots it got) or shrinks the window, keeping
 *   the copies needed soonest; waits for the copy stream and for the layers that last used the slots.
 * disable: brings every copy back to device memory of its own and releases slots and host memory.
 * ready: *ready (host) = 1 when the copy that harli_lora_fwd (backward = 0) or harli_lora_bwd (backward = 1) of `layer`
 *   needs is on the device now (always 1 without a window): what a scheduler asks before it calls the finetune task
 *   "ready" (Sec. 6.2).  Never blocks.
 * None of these may run concurrently with harli_lora_fwd / harli_lora_bwd on the same context. */
typedef struct harli_window_stats {
  int32_t slots;      /* 0 = no window */
  size_t slot_bytes;  /* one layer's frozen weights in one orientation */
  size_t host_bytes;  /* pinned host memory held */
  int64_t h2d_bytes;  /* host-to-device bytes copied so far */
  int64_t hits, misses, refills; /* acquisitions found on the device / loaded on demand; slots refilled after use */
} harli_window_stats;
harli_status harli_ft_window_enable(harli_ctx* c, int32_t n_slots);
harli_status harli_ft_window_resize(harli_ctx* c, int32_t n_slots);
harli_status harli_ft_window_disable(harli_ctx* c);
harli_status harli_ft_window_ready(harli_ctx* c, int32_t layer, int32_t backward, int32_t* ready);
harli_status harli_ft_window_stats(harli_ctx* c, harli_window_stats* out);
/* Window size for the next training step (Sec. 4.4: the finetune task hands memory to inference under pressure and takes
 * it back when chunks are free; the paper gives the behaviour, the step sizes are this library's).  Pure host
 * arithmetic, no context: call it between training steps and pass *target to harli_ft_window_resize when it differs
 * from `slots`.
 *   slots, max_slots: the window now (>= 1) and the most it may hold (>= slots).  slot_chunks: pool chunks one slot
 *   takes (slot_bytes / chunk bytes, rounded up).  free_chunks: harli_pool_stats.free_chunks now.  need_chunks: chunks
 *   the next step's saved activations and the KV reserve need free.  pressed: nonzero when inference was short of memory
 *   since the last step (harli_pool_pressure > 0) or the last training step ran out of pool memory.
 *   *calm (host, in/out, start at 0): roomy steps in a row, kept by the caller between calls.
 * Rule: slots move in groups of four.  pressed or free < need: shrink at once by ceil(max(need - free, slot_chunks) /
 * (4 slot_chunks)) groups, never under min(slots, 4), *calm = 0.  Otherwise, free > need + 8 slot_chunks and slots <
 * max_slots: ++*calm, and from the second such step in a row grow by one group (at most to max_slots).  Otherwise keep,
 * *calm = 0.  HARLI_ERR_INVALID for arguments outside these ranges. */
harli_status harli_ft_window_advise(int32_t slots, int32_t max_slots, int64_t slot_chunks, int64_t free_chunks,
                                    int64_t need_chunks, int32_t pressed, int32_t* calm, int32_t* target);

/* ======================================================================== *
 * Output layer of the finetune task with next-token cross entropy (Sec. 2.1: "output layer" after the stack of
 * transformer layers; the loss of the workloads that carry a vocabulary).  Needs g_final and w_lm in the context
 * and harli_lora_attach.
 *   h = RMSNorm(x; g_final);  logits = h W_lm^T;
 *   loss = mean over the positions with targets[i] >= 0 of  -log softmax(logits[i])[targets[i]];
 *   dx = d loss / d x   (W_lm and g_final are frozen).
 * x: device fp32 [T, hidden], the last layer's output.  targets: device int32 [T], a class index below vocab or a
 * negative value for a position that is not counted (the last token of each sequence); an index >= vocab sets the
 * context's error flag (harli_ctx_check) and the position is skipped.  loss: device fp32 scalar.  dx: device fp32
 * [T, hidden].  1 <= T <= cfg.max_ft_tokens.  Asynchronous on the stream; the library keeps half-precision copies of
 * W_lm and W_lm^T and a workspace (logits are produced in row chunks and never returned).
 * ======================================================================== */
harli_status harli_head_fwd_bwd(harli_ctx* c, const float* x, const int32_t* targets, int32_t T, float* loss, float* dx,
                                void* hip_stream);

/* ======================================================================== *
 * Adapter update (Sec. 2.1: finetuning = forward, backward, update).  The paper names no optimizer; this is
 * AdamW with decoupled weight decay over n elements, all arithmetic in fp32:
 *   g = grad[i] * grad_scale;  m = beta1*m + (1-beta1)*g;  v = beta2*v + (1-beta2)*g*g;
 *   master -= lr * ( (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps) + weight_decay * master )
 * master, m, v: device fp32 [n], updated in place (m, v start at zero).  grad: device fp32 [n] (the dA / dB that
 * harli_lora_bwd accumulated); cleared afterwards when zero_grad != 0.  param_bf16: device bfloat16 [n], rewritten
 * from master with round-to-nearest-even -- the A / B buffer given to harli_lora_attach -- or NULL (with fp32
 * storage the master itself can be the attached buffer).  step >= 1.
 * Asynchronous on the stream.  HARLI_ERR_INVALID for null pointers, step < 1 or betas outside [0, 1).
 * ======================================================================== */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay, grad_scale;
  int32_t step;      /* 1-based count of updates, for the bias corrections */
  int32_t zero_grad; /* clear grad after the update */
} harli_adamw_cfg;
harli_status harli_adamw_step(float* master, float* m, float* v, float* grad, void* param_bf16, size_t n,
                              const harli_adamw_cfg* cfg, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* HARLI_H */
