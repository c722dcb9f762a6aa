/*
 * nnc.h - C ABI of the MI355X (gfx950) Qwen3-style decoder forward pass.
 *
 * The workload is the one the nncase paper compiles and times: the decode stage
 * (and the prompt pass before it) of Qwen3-0.6B / 1.7B at batch 1, tokens/s over
 * the decoding stage (Section 4, experimental setup; Sections 4.1 and 4.2), with
 * weights laid out once, ahead of time, in the layout the matmul micro-kernel
 * wants (Section 3.1.2 "Auto Vectorize": packed / blocked layouts; Section 3.3.1:
 * constants are pre-split and pinned; Section 3.3.2: MatMul micro-kernels over
 * packed operands).  Here the packed layout is the CDNA4 matrix-core fragment
 * order and the micro-kernels are hand-written HIP.
 *
 * Conventions for every entry point
 *   - returns nnc_status; never throws, never aborts; on error the out-params and
 *     the model state are left untouched and nnc_last_error() describes the cause;
 *   - "host" pointers are ordinary CPU memory read during the call only;
 *     "device" pointers are GPU memory owned by the caller, read or written by
 *     work enqueued on the model's stream; calls do not synchronise the stream
 *     (a long prompt's last pass runs on a second stream that the library creates
 *     and joins back to the model's stream with events before the call returns,
 *     see NNC_OPT_TAIL_OVERLAP: a caller still orders its work on the one stream);
 *   - a model is bound to the GPU that was current at nnc_model_create and to one
 *     stream; calls on one model must not overlap (not thread-safe);
 *   - positions are implicit: each KV slot remembers its length, nnc_prefill and
 *     nnc_decode_step append at that length.
 *
 * Canonical weight blob (host memory, little endian, tensors contiguous,
 * matrices row-major [out, in] in blob_dtype, gains always fp32), in order:
 *   embed [V,H]                                   if has_embed_and_head
 *   per layer: g_in [H], Wq [Dq,H], Wk [Dkv,H], Wv [Dkv,H], g_q [d], g_k [d],
 *              Wo [H,Dq], g_post [H], Wgate [F,H], Wup [F,H], Wdown [H,F]
 *   g_final [H]                                   if has_embed_and_head
 *   lm_head [V,H]                                 if has_embed_and_head && !tied_lm_head
 * with Dq = n_q_heads*head_dim, Dkv = n_kv_heads*head_dim.
 * blob_dtype NNC_W8 (weight-only 8 bits; the paper has no low-bit format: this extends its
 * 16-bit runs of Section 4 towards the memory wall it names in Sections 4.1 and 4.2): every
 * matrix of a layer is [out, in] signed bytes q followed by [out] fp32 scales s, the weight being
 * s[row] * q[row][col]; embed and lm_head are bf16; hidden and ffn are multiples of 64.
 */
#ifndef NNC_H_
#define NNC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct nnc_model nnc_model; /* opaque; owned by the library */

typedef enum {
  NNC_OK = 0,
  NNC_E_ARG = 1,     /* null pointer, slot/batch/token out of range, duplicate slots */
  NNC_E_CONFIG = 2,  /* unsupported or inconsistent nnc_config */
  NNC_E_BLOB = 3,    /* blob_bytes does not match the config */
  NNC_E_NOMEM = 4,   /* device allocation failed */
  NNC_E_KV_FULL = 5, /* a slot would exceed max_seq */
  NNC_E_DEVICE = 6,  /* HIP error, or no gfx950 device */
  NNC_E_STATE = 7    /* call not valid for this model (e.g. token API on a hidden-state model) */
} nnc_status;

typedef enum {
  NNC_F32 = 0,
  NNC_BF16 = 1,
  NNC_F16 = 2, /* IEEE binary16, the paper's F16 (Section 4, setup) */
  NNC_W8 = 3   /* blob_dtype only: bytes with one scale per output row in the layers, bf16 elsewhere */
} nnc_dtype;

typedef struct {
  uint32_t struct_bytes; /* = sizeof(nnc_config) */
  uint32_t hidden, n_layers, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  float rms_eps, rope_theta;
  uint32_t has_embed_and_head; /* 0: hidden state in, hidden state out (one-layer fp32 config) */
  uint32_t tied_lm_head;       /* 1: LM head is the embedding matrix, blob holds no lm_head */
  uint32_t blob_dtype;         /* nnc_dtype of the matrices in the blob */
  uint32_t compute_dtype;      /* NNC_F32: fp32 weights, fp32 KV cache, fp32 matrix-core math;
                                  NNC_BF16 / NNC_F16: 16-bit weights and KV cache in that format,
                                  fp32 accumulation (activations enter the matrix cores as 16-bit
                                  pieces of that format).  Must equal blob_dtype, or be a 16-bit type
                                  with an NNC_F32 blob (weights are then rounded to nearest even
                                  once, at create).  An NNC_W8 blob computes in NNC_BF16: the decode
                                  GEMMs stream the bytes, widen them to bf16 exactly in registers and
                                  multiply the row sums by the scales; bf16 KV cache, embedding and
                                  LM head.  Prompt blocks widen each matrix (exactly) into a scratch
                                  matrix of bf16 tiles first and scale the rows in the GEMM's epilogue;
                                  batch-1 decode runs through the per-stage kernels (the resident decode
                                  kernel takes 16-bit weights only). */
  uint32_t max_batch;          /* number of KV slots */
  uint32_t max_seq;            /* positions per slot */
} nnc_config;

/* Device memory and stream come from the caller (e.g. PyTorch's allocator and
 * current stream).  alloc returns device memory aligned to >= 256 bytes or NULL;
 * both callbacks are invoked only inside nnc_model_create / nnc_model_destroy.
 * A NULL nnc_device, or NULL alloc/free, selects hipMalloc/hipFree and the
 * default stream. */
typedef struct {
  void *(*alloc)(size_t bytes, void *ctx);
  void (*free)(void *p, void *ctx);
  void *ctx;
  void *stream; /* hipStream_t; NULL = default stream */
} nnc_device;

/*
 * Build a model: validate the config, check blob_bytes, allocate weights / KV
 * cache / workspace, upload and repack every matrix once into the matrix-core
 * tile layout (the on-GPU counterpart of the paper's packed constant layouts,
 * Sections 3.1.2 and 3.3.1): Wq|Wk|Wv fused row-wise, Wgate/Wup interleaved in
 * 16-row tiles, bf16 rounding if requested.  blob is host memory borrowed for
 * the duration of the call.  Synchronises the stream before returning.
 */
nnc_status nnc_model_create(const nnc_config *cfg, const void *blob, size_t blob_bytes,
                            const nnc_device *dev, nnc_model **out);

/* Release everything obtained through nnc_device.alloc.  NULL is allowed.
 * Synchronises the stream first.  (Lifetime management: the paper is silent; defined here.) */
void nnc_model_destroy(nnc_model *m);

/*
 * Prompt pass (the paper's pre-decode stage, Section 4 setup): run n tokens
 * (host int32, each in [0, vocab)) through the model for one KV slot, appending
 * K/V at positions len..len+n-1.  logits_out: device, vocab floats, logits of the
 * LAST position; may be NULL.  next_out: device int32, greedy arg-max of those
 * logits (lowest index wins ties); may be NULL.  Chunked prefill = repeated calls.
 * NNC_E_KV_FULL if len + n > max_seq.
 */
nnc_status nnc_prefill(nnc_model *m, uint32_t slot, const int32_t *tokens, uint32_t n,
                       float *logits_out, int32_t *next_out);

/*
 * One decode step (the stage the paper's tokens/s metric covers): one token for
 * each of `batch` distinct slots (host arrays slots[batch], tokens[batch]).
 * logits_out: device [batch, vocab] floats or NULL.  next_out: device [batch]
 * int32 greedy tokens or NULL.
 */
nnc_status nnc_decode_step(nnc_model *m, const uint32_t *slots, const int32_t *tokens,
                           uint32_t batch, float *logits_out, int32_t *next_out);

/*
 * Greedy decode loop with the token fed back on the device: n_steps decode steps
 * for `batch` distinct slots starting from first_tokens (host), no host
 * synchronisation between steps.  tokens_out: device [n_steps, batch] int32, the
 * token produced by each step.  logits_out: device [n_steps, batch, vocab] floats
 * or NULL.  NNC_E_KV_FULL if any slot would exceed max_seq during the run.
 */
nnc_status nnc_decode_greedy(nnc_model *m, const uint32_t *slots, const int32_t *first_tokens,
                             uint32_t batch, uint32_t n_steps, int32_t *tokens_out,
                             float *logits_out);

/*
 * nnc_decode_step for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * results bit for bit as nnc_decode_step when that is called with a logits buffer (one kernel
 * per stage, launched eagerly on the model's stream), but the call allocates nothing: no
 * device or host memory, no graph, no event.  Its workspace is a fixed array of
 * NNC_STATIC_SCRATCH_MIB MiB inside the library's code object, one copy per GPU, held from
 * the first use until the process ends.
 * Limits: batch <= NNC_STATIC_MAX_BATCH, and the step's workspace (it grows with batch x
 * hidden / ffn sizes and with batch x query heads x cached positions; without logits_out also
 * batch x vocab floats) must fit the array: NNC_E_ARG with the byte counts otherwise, state
 * untouched.  NNC_E_STATE while nnc_profile_begin is active or if the model's GPU is not the
 * current device.
 * Every call on one GPU shares that GPU's array, whatever the model or stream: calls that
 * overlap on one GPU race.  Nothing in the array has to start at zero (every word a kernel
 * reads was written earlier in the same call), so no call clears it.
 */
#define NNC_STATIC_SCRATCH_MIB 24
#define NNC_STATIC_MAX_BATCH 8
nnc_status nnc_decode_step_static(nnc_model *m, const uint32_t *slots, const int32_t *tokens,
                                  uint32_t batch, float *logits_out, int32_t *next_out);

/* Forget the contents of one slot (slot >= 0) or of all slots (slot = -1): the slot's length
 * becomes 0, nothing is cleared on the device, no work is enqueued.  The paper is silent on
 * cache management (its runs are one prompt + one decode loop, Section 4 setup); defined here
 * so that one model serves request after request. */
nnc_status nnc_kv_reset(nnc_model *m, int32_t slot);

/*
 * Wait for all work enqueued on the model's stream and report deferred failures: the resident
 * decode kernel bounds every wait for an exchange word; if one ran out, all its workgroups
 * exited early, the outputs of that call are invalid and NNC_E_DEVICE is returned here and
 * by every later prompt / decode call on the model (they check without waiting).
 */
nnc_status nnc_synchronize(nnc_model *m);

/* Current length of a slot (host out-param).  (Paper silent; bookkeeping of this library.) */
nnc_status nnc_slot_len(const nnc_model *m, uint32_t slot, uint32_t *len_out);

/*
 * Hidden-state variants for models created with has_embed_and_head = 0: one decoder layer
 * (or several) without embedding and LM head, the unit the paper's operator-level
 * discussion is about (Section 3.1.2, the attention-like MatMul / Exp / MatMul chain) and the shape
 * of the smallest benchmark configuration.  The paper defines no such call; defined here.
 * x: device [n, hidden] floats in; y: device [n, hidden] floats out (the residual
 * stream after the last layer).  nnc_prefill_hidden treats the n rows as
 * consecutive positions of one slot; nnc_decode_step_hidden treats row i as the
 * next position of slots[i].
 */
nnc_status nnc_prefill_hidden(nnc_model *m, uint32_t slot, const float *x, uint32_t n, float *y);
nnc_status nnc_decode_step_hidden(nnc_model *m, const uint32_t *slots, const float *x,
                                  uint32_t batch, float *y);

/*
 * Copy cached rows out for inspection: positions pos0..pos0+n-1 of one layer and
 * slot, widened to fp32, as [n, Dkv] (kv head major inside a row) into device
 * memory `out`.  which: 0 = K (after QK-norm and RoPE), 1 = V.
 */
nnc_status nnc_kv_read(nnc_model *m, uint32_t layer, uint32_t slot, uint32_t which, uint32_t pos0,
                       uint32_t n, float *out);

/* Runtime switches. */
typedef enum {
  NNC_OPT_GRAPH = 0,        /* 1 (default): replay decode steps as captured HIP graphs; 0: eager */
  NNC_OPT_PREFILL_EXACT = 1, /* precision of the prompt pass of bf16 models.
                               0 (default): blocks of up to 4096 tokens with LDS-staged
                               matrix-core GEMMs and matrix-core attention.  Blocks of up to 512
                               tokens carry every matrix-core input as two bf16 pieces (16
                               significant bits); longer blocks round those inputs to bf16 once.
                               A call with more than 512 tokens runs its last 16 tokens through
                               the three-piece path of mode 1, so that the logits of the last
                               position see single-piece noise only through the cache; the LM
                               head itself is always fp32-grade.
                               2: the same blocks, two pieces at every length (twice the
                               matrix-core work of long blocks).
                               1: 21-token chunks through the decode kernels, three bf16 pieces
                               (fp32-grade) */
  NNC_OPT_PERSISTENT = 2,   /* 1 (default): batch-1 decode steps of bf16 models run in one
                               resident kernel per call (all steps of nnc_decode_greedy in a
                               single launch); 0: one kernel per stage */
  NNC_OPT_PREFILL_TILE = 4, /* block tile of the large-block prompt GEMMs: -1 (default) chosen from
                               each launch's size; 0: 64 x 128, 1: 256 x 128, 2: 128 x 128, 3: 64 x 64,
                               4: 192 x 128, 5: 256 x 256, 6: 192 x 256 (rows x operand columns).  Same k order per output
                               element in all, hence bit-identical results, except where the k range of
                               a narrow (residual) projection is split over several workgroups (partial
                               sums added in a fixed order): with a forced tile only the 64-row tiles do
                               that by themselves, for short blocks; see NNC_OPT_PREFILL_KSLICES */
  NNC_OPT_PREFILL_KSLICES = 13, /* with a forced NNC_OPT_PREFILL_TILE: k slices (1 .. 4) of the output and
                               down projections of a large prompt block, 0 (default): by the rule above.
                               Without a forced tile the tile model picks tile and slices together */
  NNC_OPT_PREFILL_ATTN = 6, /* launch shape of the large-block prompt attention: -1 (default) chosen
                               from each launch's size; else bit 0: every workgroup takes a long
                               and a short 64-token block, bit 1: two query heads per wave; results
                               are bit-identical for all (a wave's arithmetic per head is the same) */
  NNC_OPT_FUSE_QK = 7,      /* 1 (default): per-stage decode passes of bf16 models do QK-norm, RoPE and
                               the cache append inside the attention kernel (one kernel less per
                               layer); 0: in a kernel of their own.  Bit-identical results */
  NNC_OPT_TAIL_OVERLAP = 8, /* 1 (default): the fp32-grade pass over the last tokens of a long prompt is
                               enqueued on a second stream of the library's own and runs beside the
                               prompt's last block, each of its layers waiting (event) for that
                               layer's cache rows; the model's stream waits for it before the call
                               returns to the caller's later work.  0: it follows the block on the
                               model's stream.  Bit-identical results */
  NNC_OPT_PREFILL_BLOCK = 9, /* tokens per block of the large-block prompt pass: 0 (default) = the largest
                               (4096, or max_seq rounded up to 128 if that is less); else a multiple of
                               128.  Longer blocks give the narrow projections enough workgroups for the
                               largest block tile; the blocking does not change which inputs are rounded
                               (every block of more than 512 tokens carries one bf16 piece) */
  NNC_OPT_PLANNER = 10,     /* 1 (default): block tiles, row tiles per workgroup and k slices of the GEMM
                               launches come from the analytic model behind nnc_plan_*_query; 0: from the
                               hand-written rules that preceded it (kept for comparison) */
  NNC_OPT_FUSE_NORM = 11,   /* 1: in per-stage decode passes the RMSNorm after an output / down
                               projection runs in the tail of that GEMM launch (its last workgroups to
                               finish wait for the others, one per sequence, and norm the rows): two
                               kernels less per layer, same arithmetic, bit-identical results; the wait
                               is bounded by NNC_OPT_SPIN_LIMIT.  0 (default): in a kernel of its own --
                               the hand-over inside the launch (store acknowledgement, counter, reads
                               past the caches) takes as long as the kernel boundary it replaces */
  NNC_OPT_DECODE_PIECES = 12, /* bf16 / binary16 pieces an activation is split into before a decode GEMM of
                               a batch of two or more sequences: 0 (default) the library's choice, 2 or 3
                               forced.  Three pieces carry an fp32 value to 2^-25 relative, two to 2^-17
                               (a third fewer operand columns) */
  NNC_OPT_SPIN_LIMIT = 5,   /* polls after which a wait inside the resident kernel gives up (sets
                               the failure flag and lets every workgroup exit); 0 (default):
                               2^20, about a second.  A tiny value makes the give-up path testable */
  NNC_OPT_STAGE_TRACE = 3   /* s + 1: the resident kernel stamps the 100 MHz wall clock at every
                               stage boundary of decode step s of each following launch (read them
                               with nnc_stage_trace); 0 (default): off */
} nnc_option;
nnc_status nnc_set_option(nnc_model *m, nnc_option opt, int32_t value);

/*
 * Per-kernel timing with HIP events on the model's stream.  After
 * nnc_profile_begin, every launch of the forward pass runs eagerly and is
 * bracketed by events; nnc_profile_end synchronises, stops profiling and fills up
 * to `cap` records (host), returning the number written in *n_out.
 */
typedef struct {
  char name[48];        /* kernel family, e.g. "attn_partial"; the skinny GEMM reports one record per
                           matrix it streams: "gemm_skinny.qkv", ".o", ".gate_up", ".down", ".lm_head" */
  uint64_t launches;
  double total_ms;      /* sum of event-to-event times */
  double bytes;         /* algorithmic bytes those launches had to move */
  double flops;         /* algorithmic flops (2 per multiply-add) */
} nnc_kernel_stat;
nnc_status nnc_profile_begin(nnc_model *m);
nnc_status nnc_profile_end(nnc_model *m, nnc_kernel_stat *out, uint32_t cap, uint32_t *n_out);

/*
 * Stage stamps of the last traced resident-kernel launch (see NNC_OPT_STAGE_TRACE), for
 * tuning: host buffer out[workgroups][points] of 64-bit wall-clock ticks (10 ns each).
 * Per layer 8 points: layer start, QKV operand ready, q|k|v published, attention partials
 * published, attention block output published, gate/up operand ready, activations
 * published, MLP output published; then LM-head operand ready, per-workgroup winners
 * published, token known.  Synchronises the stream.  NNC_E_ARG if cap (in
 * 64-bit words) is too small; NNC_E_STATE if tracing is off.
 */
nnc_status nnc_stage_trace(nnc_model *m, uint64_t *out, uint32_t cap, uint32_t *workgroups,
                           uint32_t *points);

/*
 * The analytic tile chooser the library plans its GEMM launches with, exposed for inspection and
 * tests (host code only, no GPU needed).  It follows the paper's parametric optimisation
 * (Section 3.2.2): tile variables, capacity constraints per storage level (LDS bytes of the
 * staged operands, registers per wave), and the objective minimise max(T_mem, T_comp) with T_comp
 * from a linear regression of the micro-kernel's time per k step and T_mem = traffic / bandwidth,
 * plus launch and epilogue-traffic time.  The search space is the block tiles the kernels are
 * instantiated for, times the k slices a launch may use, so the problem is solved by enumeration.
 * epilogue: 0 store, 1 add to the residual stream, 2 SwiGLU.  n_cus: compute units (0 = 256).
 *   nnc_plan_prefill_gemm_query  prompt GEMM [rows x k] x [k x n_tokens] with `pieces` 16-bit
 *                                pieces per activation; may use up to max_k_slices k slices
 *   nnc_plan_skinny_gemm_query   weight-streaming GEMM of a decode pass with n_seq sequences of
 *                                `pieces` pieces each; T_mem has two levels here: t_mem_us = the
 *                                weights from HBM, t_comp_us = what the busiest compute unit moves
 *                                through its vector memory path (its workgroups' weight tiles and
 *                                operand reads); tile_rows = rows per workgroup (16 x 1, 2, 3, 4, 6
 *                                or 8 row tiles); max_k_slices = partial sums the consumer can add
 */
typedef struct {
  uint32_t tile_rows, tile_cols;  /* block tile (rows x operand columns) */
  int32_t tile_code;              /* the library's code of that tile (NNC_OPT_PREFILL_TILE) / row tiles per workgroup */
  uint32_t k_slices, workgroups;
  double t_comp_us, t_mem_us, t_us; /* model times of the choice */
  uint32_t candidates, rejected_by_capacity; /* prompt GEMM: tiles enumerated / ruled out by LDS or registers */
} nnc_gemm_plan;
nnc_status nnc_plan_prefill_gemm_query(uint32_t rows, uint32_t k, uint32_t n_tokens, uint32_t pieces,
                                       uint32_t epilogue, uint32_t max_k_slices, uint32_t n_cus,
                                       nnc_gemm_plan *out);
nnc_status nnc_plan_skinny_gemm_query(uint32_t rows, uint32_t k, uint32_t n_seq, uint32_t pieces,
                                      uint32_t epilogue, uint32_t max_k_slices, uint32_t n_cus,
                                      nnc_gemm_plan *out);

/* Bytes of the canonical blob for a config (0 if the config is invalid).  (Paper silent: the blob
 * is this library's input format, the stand-in for the paper's pre-laid-out constants,
 * Section 3.3.1.) */
uint64_t nnc_blob_bytes(const nnc_config *cfg);

/* Message for the most recent failure on this thread (static storage).  (Paper silent.) */
const char *nnc_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* NNC_H_ */
