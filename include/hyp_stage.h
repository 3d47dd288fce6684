/*
 * hyp_stage.h - C ABI of the stage-forward library for AMD MI355X (gfx950).
 *
 * A *stage* is the unit of work that the paper's pipeline hands to one node: the
 * contiguous range of decoder blocks I_j(p) = { i : p_{j-1} < i <= p_j } (Eq. 6),
 * executed in strict order (Eq. 1) on the activation tensor
 * batch x sequence x hidden that travels between tiers (Sec. IV-A).  Every block
 * is the one of Sec. III-A / Fig. 2: RMS Norm -> grouped-query attention with
 * rotary position encoding -> residual, RMS Norm -> SwiGLU feed-forward ->
 * residual.  Requests are first *prefilled* (the whole prompt) and then *decoded*
 * one token per step against the keys and values cached at prefill (the
 * experiments of Sec. V-A use 64 prompt tokens and 128 or 256 generated ones,
 * with weights and caches resident while generating, Sec. V-D).
 *
 * Conventions the paper leaves open and this library fixes (the CPU oracle used
 * by the tests fixes the same ones):
 *   - pre-norm residuals around both sub-layers; eps is added to the mean square
 *     inside the square root; there are no biases;
 *   - RoPE pairs element i with i + head_dim/2 of every query and key head
 *     (rotate-half) and turns the pair by pos * rope_base^(-2i/head_dim);
 *   - query head h reads KV head h / (n_q_heads / n_kv_heads);
 *   - scores are scaled by 1/sqrt(head_dim); a query at position p sees keys at
 *     positions 0..p and nothing else;
 *   - prefill token t of a request sits at position t; a decode token sits at
 *     the position equal to the number of tokens already cached;
 *   - [l_start, l_end) is the 0-based half-open form of the paper's 1-based
 *     (p_{j-1}, p_j].
 *
 * All pointers are plain addresses.  "device" = memory of the current HIP device
 * that the caller owns (e.g. a PyTorch tensor's storage) and keeps alive for the
 * time stated; "host" = ordinary process memory.  No call allocates or frees
 * device memory: the caller supplies one workspace.  No call throws (C++ exceptions
 * are caught at the boundary and become HYP_ENOMEM / HYP_EDEVICE), aborts or
 * prints; every failure is a status code plus a message from stage_last_error().
 * A stage is not thread-safe; use one stage per host thread or lock outside.
 */
#ifndef HYP_STAGE_H
#define HYP_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HYP_API __attribute__((visibility("default")))

typedef struct hyp_stage hyp_stage_t; /* opaque */

typedef enum {
  HYP_OK = 0,
  HYP_EINVAL = 1,    /* null pointer, bad layer range, bad enum                  */
  HYP_ESHAPE = 2,    /* shape the block definition does not admit                */
  HYP_ECAPACITY = 3, /* batch / sequence / token count beyond what was configured */
  HYP_ESTATE = 4,    /* call out of order (decode before prefill, ...)           */
  HYP_EDEVICE = 5,   /* a HIP call failed; text in stage_last_error()            */
  HYP_ENOMEM = 6     /* workspace too small / host allocation failed             */
} hyp_status_t;

typedef enum { HYP_F32 = 0, HYP_BF16 = 1 } hyp_dtype_t;

/* hyp_stage_config_t.flags */
#define HYP_FLAG_NO_GRAPH 2u      /* launch the decode-step kernels one by one instead of replaying \
                                     a recorded HIP graph                                 */
#define HYP_FLAG_PAGED_KV 4u      /* keep the KV cache in pages of HYP_KV_PAGE_KEYS keys addressed through a \
                                     page table (stage_set_page_table) instead of one slab per request; \
                                     stages on the MFMA kernels only                                   */
#define HYP_KV_PAGE_KEYS 128
#define HYP_FLAG_PLAIN_KERNELS 1u /* diagnostics: run the shape-generic HIP kernels even \
                                     where the MFMA kernels apply                        */

typedef struct {
  int32_t hidden;       /* H                                                  */
  int32_t n_q_heads;    /* query heads                                        */
  int32_t n_kv_heads;   /* key/value heads; must divide n_q_heads             */
  int32_t head_dim;     /* d, even                                            */
  int32_t ffn_dim;      /* SwiGLU inner width I                               */
  float rms_eps;
  float rope_base;
  int32_t dtype;        /* hyp_dtype_t: type of weights, activations and cache */
  int32_t max_batch;    /* requests resident at once                          */
  int32_t max_seq;      /* per-request capacity: prompt + generated tokens    */
  int64_t max_prefill_tokens; /* bound on sum(seq_lens) of one stage_prefill   */
  uint32_t flags;
  uint32_t kv_pool_pages; /* HYP_FLAG_PAGED_KV: pages in the pool of every block; 0 = enough for
                             max_batch requests of max_seq keys.  Must be 0 without the flag.   */
} hyp_stage_config_t;

/* Weights of one block: device pointers, row-major [out_features, in_features]
 * (y = x W^T), type = config dtype.  Read during stage_create only. */
typedef struct {
  const void *attn_norm_g; /* [hidden]                       */
  const void *wq;          /* [n_q_heads*head_dim, hidden]   */
  const void *wk;          /* [n_kv_heads*head_dim, hidden]  */
  const void *wv;          /* [n_kv_heads*head_dim, hidden]  */
  const void *wo;          /* [hidden, n_q_heads*head_dim]   */
  const void *ffn_norm_g;  /* [hidden]                       */
  const void *w_gate;      /* [ffn_dim, hidden]              */
  const void *w_up;        /* [ffn_dim, hidden]              */
  const void *w_down;      /* [hidden, ffn_dim]              */
} hyp_layer_weights_t;

/* Bytes of device workspace stage_create needs for this configuration and layer
 * range (weights in the library's own layout, KV cache, position tables,
 * scratch).  Returns 0 if the arguments are invalid. */
HYP_API size_t stage_workspace_bytes(const hyp_stage_config_t *cfg, int32_t l_start, int32_t l_end);

/* Build the stage that owns blocks [l_start, l_end) (Eq. 6).
 *   layers     host array of l_end - l_start weight records (device pointers
 *              inside); record i belongs to block l_start + i.
 *   workspace  device, >= stage_workspace_bytes(), 256-byte aligned, owned by the
 *              caller and kept alive and untouched until stage_destroy.
 *   hip_stream a hipStream_t (0 = the null stream), borrowed; every later call on
 *              this stage enqueues its work there.
 * The weights are copied into the workspace in the library's layout and the
 * call returns only after that copy has finished, so the caller may release the
 * original weight tensors afterwards.
 * Errors: HYP_EINVAL (null pointer, l_start < 0, l_start >= l_end, bad dtype, unknown
 * flag, kv_pool_pages without HYP_FLAG_PAGED_KV), HYP_ESHAPE (non-positive size, n_q_heads % n_kv_heads != 0, odd
 * head_dim), HYP_ENOMEM (workspace too small or misaligned), HYP_EDEVICE. */
HYP_API hyp_status_t stage_create(const hyp_stage_config_t *cfg, int32_t l_start, int32_t l_end,
                          const hyp_layer_weights_t *layers, void *workspace,
                          size_t workspace_bytes, void *hip_stream, hyp_stage_t **out);

/* Prefill: run the stage's blocks over the prompts of `batch` requests and fill
 * their KV cache (Sec. III-A block, Eq. 1 order; the input is the activation
 * tensor of Sec. IV-A, i.e. hidden states, also for the first stage).
 *   hidden_in  device, [sum(seq_lens), hidden] row-major, requests packed one
 *              after the other without padding; read-only.
 *   seq_lens   host, [batch], each in 1..max_seq; read before the call returns.
 *   hidden_out device, same shape and type; may be the same buffer as hidden_in.
 * Any earlier requests of the stage are dropped: request b of this call
 * becomes slot b.  The work is enqueued on the stage's stream; the call does not
 * wait for it.
 * Errors: HYP_EINVAL (null), HYP_ECAPACITY (batch < 1 or > max_batch, a length
 * outside 1..max_seq, sum > max_prefill_tokens), HYP_EDEVICE.  On error the
 * stage keeps its previous requests. */
HYP_API hyp_status_t stage_prefill(hyp_stage_t *stage, const void *hidden_in, const int32_t *seq_lens,
                           int32_t batch, void *hidden_out);

/* One decode step: one new token for every resident request, at the position
 * equal to its cached length; its key and value are appended to the cache
 * (KV-cached generation, Sec. V-A workload).
 *   hidden_in / hidden_out  device, [batch, hidden]; may alias.
 * Asynchronous on the stage's stream.
 * Errors: HYP_ESTATE (no prefill yet), HYP_ECAPACITY (some request already holds
 * max_seq tokens; nothing is changed), HYP_EINVAL, HYP_EDEVICE. */
HYP_API hyp_status_t stage_decode_step(hyp_stage_t *stage, const void *hidden_in, void *hidden_out);

/* stage_decode_step for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Same arguments, same result bit for bit, but
 * the step's temporaries (partial sums and arrival counters of the split GEMVs, per-chunk
 * attention results, the block's activations of the <= 32 tokens) live in a 32 MiB array that is
 * part of the library's device image instead of the workspace, the kernels are launched one by
 * one (no graph is recorded or instantiated), no events are created, and the call performs no
 * device or host allocation.  Every stage and every call on one GPU shares that GPU's array:
 * calls that overlap on one GPU (two streams, two threads) race; calls ordered on one stream or
 * by events are fine.  Serves stages that run the MFMA kernels (stage_uses_mfma).
 * Errors: as stage_decode_step, plus HYP_ESHAPE (stage on the shape-generic kernels) and
 * HYP_ECAPACITY when one step's temporaries exceed the array (the Phi-3-medium-shaped and
 * Llama3-8B-shaped blocks at up to 32 requests fit); nothing is changed then. */
HYP_API hyp_status_t stage_decode_step_noalloc(hyp_stage_t *stage, const void *hidden_in, void *hidden_out);

/* Paged KV cache ("weights and associated caches" stay resident on the node, Sec. V-D; with
 * pages a request only occupies the keys it holds, so more requests fit one node's memory).
 * A stage created with HYP_FLAG_PAGED_KV stores keys and values in a pool of pages of
 * HYP_KV_PAGE_KEYS keys per block of the stage; this call says which pages the request slots use:
 *   table  host, [n_requests][pages_per_request]: table[r][i] is the pool page (0 <=
 *          page < kv_pool_pages, the same in every block of the stage) that holds keys
 *          [128 i, 128 i + 128) of request slot r, or -1 for none; no page may appear twice.
 *          Slots >= n_requests and columns >= pages_per_request get no page.  Copied before
 *          the call returns (the call waits for the stage's stream).
 * It applies to the prefill and decode calls that follow; pages that already hold cached keys
 * of a resident request must keep their place (HYP_ESTATE otherwise).  Without this call,
 * slot r owns pages r * ceil(max_seq / 128) ... when the pool has max_batch * ceil(max_seq /
 * 128) pages; a smaller pool starts with no pages assigned.  stage_prefill and
 * stage_decode_step return HYP_ECAPACITY, changing nothing, when a request has no page for a
 * key they would write (a prompt is written up to the next multiple of 64 keys).
 * Errors: HYP_EINVAL (null, counts < 1, page outside the pool or assigned twice),
 * HYP_ECAPACITY (n_requests > max_batch, a page beyond max_seq), HYP_ESTATE (stage without
 * the flag, or see above), HYP_EDEVICE. */
HYP_API hyp_status_t stage_set_page_table(hyp_stage_t *stage, const int32_t *table, int32_t n_requests,
                                          int32_t pages_per_request);

/* Copy the cached keys (post-RoPE) and values of one request and one block of
 * the stage (layer in [0, l_end - l_start)) to k_out / v_out, device,
 * [context_len, n_kv_heads*head_dim] row-major in the stage dtype.  This is what
 * a request needs to move to another node of the same tier.  Asynchronous.
 * Errors: HYP_EINVAL, HYP_ESTATE (no such request). */
HYP_API hyp_status_t stage_export_kv(hyp_stage_t *stage, int32_t layer, int32_t request, void *k_out,
                             void *v_out);

/* Tokens cached for `request` (host value, counts enqueued steps). */
HYP_API hyp_status_t stage_context_len(const hyp_stage_t *stage, int32_t request, int32_t *len_out);

/* Release host state.  The workspace returns to the caller, who must first
 * synchronise the stream.  stage_destroy(NULL) is HYP_EINVAL, and so is a pointer that
 * is not a live handle of this library (e.g. a stage destroyed twice): every entry
 * point checks its handle against the set of live stages before touching it. */
HYP_API hyp_status_t stage_destroy(hyp_stage_t *stage);

/* Message of the last failing call on this stage (or, with stage == NULL, of the
 * last failing stage_create / stage_workspace_bytes on this thread).  Owned by
 * the library, valid until the next call; never NULL. */
HYP_API const char *stage_last_error(const hyp_stage_t *stage);

/* Kernel classes of the MFMA path, for stage_profile(). */
typedef enum {
  HYP_K_ADD_NORM = 0,       /* residual add + RMS Norm (prefill and decode)        */
  HYP_K_GEMM_QKV = 1,       /* prefill QKV projection + RoPE + cache write         */
  HYP_K_ATTN_PREFILL = 2,   /* causal GQA attention over the prompt                */
  HYP_K_GEMM_O = 3,         /* prefill attention output projection                 */
  HYP_K_GEMM_GATEUP = 4,    /* prefill gate/up projection + SwiGLU                 */
  HYP_K_GEMM_DOWN = 5,      /* prefill down projection                             */
  HYP_K_GEMV_QKV = 6,       /* decode QKV projection (weight streaming)            */
  HYP_K_DEC_QKV_FINISH = 7, /* decode RoPE + cache append                          */
  HYP_K_ATTN_DECODE = 8,    /* decode attention over the cache + chunk merge       */
  HYP_K_GEMV_O = 9,
  HYP_K_GEMV_GATEUP = 10,
  HYP_K_DEC_SWIGLU = 11,
  HYP_K_GEMV_DOWN = 12,
  HYP_K_COUNT = 13
} hyp_kernel_class_t;

/* Measurement aid: from now on bracket every launch of the kernel classes in
 * class_mask (bit i = class i) with a pair of HIP events on the stage's stream;
 * 0 switches it off.  Either way the stream is synchronised and earlier records
 * are dropped.  Host state only (events); no device memory is allocated. */
HYP_API hyp_status_t stage_profile(hyp_stage_t *stage, uint32_t class_mask);

/* Synchronise the stream and return the summed duration (milliseconds) and the
 * number of launches of one kernel class recorded since stage_profile(). */
HYP_API hyp_status_t stage_profile_read(hyp_stage_t *stage, int32_t kernel_class, double *total_ms,
                                int64_t *launches);

/* Measurement aids: ceilings of the device measured in place, to set beside the
 * datasheet peaks in a roofline.  Neither needs a stage; both time three launches
 * with HIP events on `hip_stream` and wait for them.
 *   hyp_measure_mfma_ceiling     bf16 MFMA rate (TFLOP/s) of a register-only loop on every
 *       SIMD.  mode bit 0: operands N(0,1) (set) or the constant 1.0 (clear); mode bit 1:
 *       v_mfma_f32_32x32x16_bf16 (set; the attention kernels' instruction) or
 *       v_mfma_f32_16x16x32_bf16 (clear; the prefill GEMM's).  scratch: device, 16-byte
 *       aligned, >= 2.2 MB, overwritten.
 *   hyp_measure_hbm_read_ceiling rate (GB/s) of a plain streaming read of `buffer`
 *       (device, 16-byte aligned, >= 1 GiB - well beyond the 256 MB memory-side cache;
 *       its last 16 bytes may be overwritten).
 * Errors: HYP_EINVAL (null / too small / misaligned), HYP_EDEVICE. */
HYP_API hyp_status_t hyp_measure_mfma_ceiling(void *scratch, size_t scratch_bytes, int32_t mode,
                                      void *hip_stream, double *tflops_out);
HYP_API hyp_status_t hyp_measure_hbm_read_ceiling(const void *buffer, size_t bytes, void *hip_stream,
                                          double *gbs_out);

/* 1 if the MFMA kernels run for this stage, 0 if the shape-generic kernels do
 * (fp32 stages, head_dim != 128, widths that are not multiples of 256, or
 * HYP_FLAG_PLAIN_KERNELS). */
HYP_API int32_t stage_uses_mfma(const hyp_stage_t *stage);

#ifdef __cplusplus
}
#endif
#endif /* HYP_STAGE_H */
