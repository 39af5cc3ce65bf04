/*
 * flashformer.h -- C ABI of the MI355X whole-model decode library.
 *
 * One call to ff_decode_step runs one forward step of a Llama-style decoder (paper Section 2.1:
 * pre-RMSNorm, grouped-query attention with RoPE, SwiGLU FFN) for a batch of independent sequences
 * in ONE persistent kernel launch covering all layers (paper abstract and Section 4: a single
 * kernel invocation per generated token), followed inside the same launch by the final norm and the
 * LM head.  ff_decode_step_perop runs the same step as one launch per operation on the same
 * buffers (the paper's "Baseline": separate kernel launches, as in the latency tables of Sections 3 and 5.3).
 *
 * Conventions
 *   - Every pointer named *_dev is DEVICE memory on the current HIP device; it is allocated and
 *     owned by the caller (the library never allocates or frees device memory).  Sizes come from
 *     the *_bytes queries.  All device buffers must be 256-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls that take a
 *     stream are asynchronous on it.
 *   - Every function returns FF_OK (0) or a negative FF_ERR_* code; ff_last_error() returns a
 *     thread-local description of the last failure.  No exception crosses this boundary.
 *   - Canonical (caller-side) layouts: every projection matrix is row-major [out, in].
 *       FF_W_BF16      : bf16 [N][K]
 *       FF_W_INT8_PC   : int8 [N][K] codes, fp16 scale s[N];            w = q * s[n]
 *       FF_W_INT4_G128 : uint8 [N][K/2], two codes per byte, low nibble = even k,
 *                        fp16 s[N][K/128], fp16 z[N][K/128] (integer valued, 0..15);
 *                        w = (code - z[n][k/128]) * s[n][k/128]
 *     Norm gains and the embedding table are bf16.  The library repacks these into a private
 *     tile order inside `packed_dev`; the caller may free the canonical tensors after loading.
 */
#ifndef FLASHFORMER_H
#define FLASHFORMER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ff_model ff_model;
typedef struct ff_kv ff_kv;

enum {
    FF_OK = 0,
    FF_ERR_ARG = -1,         /* null pointer, batch outside [1, max_batch], bad index */
    FF_ERR_UNSUPPORTED = -2, /* configuration has no compiled kernel instance */
    FF_ERR_RANGE = -3,       /* a position outside [0, max_ctx), or a token id that is neither in [0, vocab) nor FF_TOKEN_SKIP (seen on device) */
    FF_ERR_NOMEM = -4,       /* a caller-provided buffer is too small or misaligned */
    FF_ERR_TIMEOUT = -5,     /* a workgroup gave up waiting for another one's output (not co-resident?) */
    FF_ERR_HIP = -6          /* a HIP runtime call failed; text in ff_last_error() */
};

enum { FF_W_BF16 = 0, FF_W_INT8_PC = 1, FF_W_INT4_G128 = 2 };

/* Token id of a sequence that takes no part in a decode step (it has stopped early while the rest
 * of the batch decodes on; the paper's batches advance in lock step, Section 5.2). */
#define FF_TOKEN_SKIP (-1)

/* Which matrix ff_debug_dequant exports. */
enum { FF_MAT_WQ = 0, FF_MAT_WK, FF_MAT_WV, FF_MAT_WO, FF_MAT_WGATE, FF_MAT_WUP, FF_MAT_WDOWN, FF_MAT_LMHEAD };

/* Model dimensions (paper Section 2.1, model-configuration table) and weight format. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rms_eps, rope_theta;
    int32_t wdtype;        /* FF_W_* for the seven per-layer projections */
    int32_t max_batch;     /* largest batch any step will use (1..16) */
    int32_t quant_lm_head; /* nonzero: LM head uses wdtype too; zero: LM head is bf16 */
} ff_config;

/* One projection matrix in canonical layout (device pointers; s/z NULL when unused). */
typedef struct {
    const void *w, *s, *z;
} ff_matrix;

typedef struct {
    const void *attn_norm, *ffn_norm; /* bf16 [d_model] */
    ff_matrix wq, wk, wv, wo, w_gate, w_up, w_down;
} ff_layer_weights;

typedef struct {
    const void *embed;      /* bf16 [vocab][d_model] */
    const void *final_norm; /* bf16 [d_model] */
    ff_matrix lm_head;      /* [vocab][d_model] */
} ff_head_weights;

const char *ff_last_error(void);

/* Bytes the caller must provide for the repacked parameters and for the activation-exchange /
 * synchronisation scratch of a model with this configuration. */
int ff_model_bytes(const ff_config *cfg, size_t *packed_bytes, size_t *scratch_bytes);

/* Creates a model over caller-owned device buffers (contents of packed_dev undefined until the
 * load calls below have run; scratch_dev is cleared here on `stream`).  FF_ERR_NOMEM if a buffer
 * is smaller than ff_model_bytes reports, FF_ERR_UNSUPPORTED for dimensions without a kernel
 * instance: (head_dim, n_q_heads / n_kv_heads) must be (64, 4), (128, 4) or (128, 8); d_model,
 * n_q_heads * head_dim and d_ffn multiples of 8 (bf16), 16 (int8) or 128 (int4);
 * d_model * 4 bytes * min(max_batch, 4) <= 128 KiB (a normalised input row is held on chip whole);
 * d_model <= 8192 when max_batch > 1. */
int ff_model_create(const ff_config *cfg, void *packed_dev, size_t packed_bytes, void *scratch_dev,
                    size_t scratch_bytes, void *stream, ff_model **out);

/* Repack one layer / the head from canonical layout into the model (device-to-device on `stream`).
 * Layers may be loaded in any order, one at a time, so a caller can generate, load and free a
 * layer at a time for models whose canonical copy would not fit beside the packed one. */
int ff_model_load_layer(ff_model *m, int32_t layer, const ff_layer_weights *w, void *stream);
int ff_model_load_head(ff_model *m, const ff_head_weights *w, void *stream);

/* Convenience: create + load every layer (layers = host array [n_layers]) + head. */
int ff_model_load(const ff_config *cfg, const ff_layer_weights *layers, const ff_head_weights *head,
                  void *packed_dev, size_t packed_bytes, void *scratch_dev, size_t scratch_bytes,
                  void *stream, ff_model **out);

/* Creates a model (as ff_model_create) and fills it on the device with the seeded synthetic weights
 * of this package's input generators (paper_2505_22758_amd/synth.py is the definition: a counter
 * hash of (seed, tensor name, element index); bf16 tensors ~N(0, 0.02), gains 1 + N(0, 0.02), int8
 * codes uniform in [-127, 127] with fp16 row scales, int4 codes and zeros uniform in [0, 15] with
 * fp16 group scales).  Bit-identical to generating the canonical tensors with synth.py and loading
 * them with ff_model_load (tested); several hundred times faster for the 139 GB 70B shape. */
int ff_model_load_synthetic(const ff_config *cfg, uint64_t seed, void *packed_dev, size_t packed_bytes,
                            void *scratch_dev, size_t scratch_bytes, void *stream, ff_model **out);
int ff_model_free(ff_model *m);

/* KV cache for `batch` independent sequences of at most max_ctx positions (paper Section 5.2:
 * caches are distinct per sequence).  bf16; keys are stored rotated.  Also holds the RoPE
 * cos/sin table for positions [0, max_ctx), built here on `stream`. */
int ff_kv_bytes(const ff_model *m, int32_t batch, int32_t max_ctx, size_t *bytes);
int ff_kv_alloc(ff_model *m, int32_t batch, int32_t max_ctx, void *kv_dev, size_t bytes, void *stream,
                ff_kv **out);
/* Copy n cache rows [pos0, pos0+n) of (layer, seq) from / to canonical bf16 [n][n_kv_heads][head_dim]. */
int ff_kv_fill(ff_kv *kv, int32_t layer, int32_t seq, int32_t pos0, int32_t n, const void *k_dev,
               const void *v_dev, void *stream);
int ff_kv_read(ff_kv *kv, int32_t layer, int32_t seq, int32_t pos0, int32_t n, void *k_dev, void *v_dev,
               void *stream);
/* Fills rows [0, n_ctx) of every (layer, sequence) with the seeded synthetic prefill of synth.py
 * (~N(0, 1) in bf16, taken as already rotated keys); same bits as ff_kv_fill of make_kv_prefill. */
int ff_kv_fill_synthetic(ff_kv *kv, uint64_t seed, int32_t n_ctx, void *stream);
int ff_kv_free(ff_kv *kv);

/* One decode step (paper Section 4.2, attention and GLU schedules; final norm and LM head added).
 *   tokens_dev    int32 [batch]   token ids, each in [0, vocab), or FF_TOKEN_SKIP: that sequence sits
 *                                 this step out -- its position is ignored, nothing is appended to
 *                                 its cache and its row of logits_dev is not written.  (Its slot
 *                                 still travels through the kernel as a placeholder, so the step
 *                                 costs what the full batch costs; the other sequences' results are
 *                                 bit-identical to a step in which it takes part.)
 *   positions_dev int32 [batch]   number of rows already cached for each sequence (= the position
 *                                 of this token); this step appends K,V at that row and attends to
 *                                 rows 0..position inclusive.  The caller advances positions.
 *   logits_dev    fp32  [batch][vocab]   valid once `stream` has synchronised.
 * Asynchronous; an out-of-range position or token anywhere in the batch makes every kernel of the
 * step skip its work (all passes: nothing is appended, and logits_dev is not written unless the LM
 * head has a weight type of its own and runs as separate launches) and record FF_ERR_RANGE in the
 * model's status word (see ff_status).  Steps on one model must not overlap.
 * A step's launches carry no host-side per-step state (exchange tags and write counters derive
 * from a counter in the model's scratch), so a step may be recorded into a HIP graph and replayed.
 * One kernel pass serves up to 4 sequences (paper Section 5.2: batches 2-4 replicate the inputs and
 * read every weight once); with max_batch > 4, batches of 5 to 16 run as ONE "wide" pass (the paper
 * stops at 4): projections on 16x16x32 matrix-core tiles (int8 and int4 codes converted to bf16 in
 * registers), activations exchanged in the consumers' on-chip layout by the workgroups that own them,
 * preceded by a small launch that prepares the step's embedding rows.  The wide pass needs the LM head
 * in the layers' format (quant_lm_head for int8 / int4) and, for int4, d_model, n_q_heads * head_dim
 * and d_ffn multiples of 512; otherwise a batch above 4 runs as consecutive passes of 4 on the
 * stream, each streaming the weights again. */
int ff_decode_step(ff_model *m, const int32_t *tokens_dev, const int32_t *positions_dev, ff_kv *kv,
                   float *logits_dev, int32_t batch, void *stream);

/* For callers that cannot allocate device memory or bring a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation): the same step as ff_decode_step, with the
 * activation-exchange scratch taken from an array of FF_STATIC_SCRATCH_BYTES that is built into the
 * library's device code (one copy per GPU, held until the process ends) instead of the model's
 * scratch_dev; only the model's status word is still used.  Calls no allocating routine.  The
 * array is shared by every model and call on the GPU and is re-initialised on `stream` at the
 * start of each call (two small extra launches), so calls need not follow each other on the same
 * model -- but two calls that overlap in time on one GPU race on it and give undefined results.
 * FF_ERR_NOMEM if the configuration's scratch (ff_model_bytes) exceeds the array: it holds the tiny
 * shape at any batch, the 8B shape up to max_batch 2 and the 70B shape at max_batch 1. */
#define FF_STATIC_SCRATCH_BYTES (8u << 20)
int ff_decode_step_static(ff_model *m, const int32_t *tokens_dev, const int32_t *positions_dev, ff_kv *kv,
                          float *logits_dev, int32_t batch, void *stream);

/* Same step as separate per-operation launches (baseline of the paper's latency tables).  After a
 * range error the cache is unchanged and logits_dev holds undefined values. */
int ff_decode_step_perop(ff_model *m, const int32_t *tokens_dev, const int32_t *positions_dev, ff_kv *kv,
                         float *logits_dev, int32_t batch, void *stream);

/* Synchronises `stream`, returns the device status word (FF_OK, FF_ERR_RANGE or FF_ERR_TIMEOUT)
 * recorded by the steps so far, and clears it.  A step that saw FF_ERR_RANGE was skipped as a whole
 * and leaves model and cache unchanged.  After FF_ERR_TIMEOUT a step has stopped half-way: the
 * model's exchange buffers are then undefined and the model must be created again. */
int ff_status(ff_model *m, void *stream);

/* Writes matrix `which` (FF_MAT_*) of `layer` (ignored for FF_MAT_LMHEAD) as fp32, canonical
 * [N][K] order, dequantised element by element from the PACKED copy by the defining formula
 * (q * s, (code - z) * s).  This checks the packing; the decode kernels never form single weights
 * (they scale finished sums), so their arithmetic is exported by ff_debug_gemv below. */
int ff_debug_dequant(const ff_model *m, int32_t layer, int32_t which, float *out_dev, void *stream);

/* Runs the decode kernels' own projection code on caller input: out_dev[b][n] = sum_k W[n][k] *
 * in_dev[b][k] for matrix `which` of `layer`, fp32 in_dev [batch][K], fp32 out_dev [batch][N] with
 * rows in canonical order.  path 0: the vector-ALU streaming GEMV (batch 1..4) used at batch 1 and
 * by the per-operation baseline; path 1: the matrix-core GEMV of batches >= 2 (batch 2..4, input
 * staged as bf16 head + remainder; K * 4 bytes * batch must fit the 128 KiB input buffer).  Fed with
 * unit vectors it returns the columns of W exactly as the hot path dequantises them (the int8 row
 * scale and the int4 group scale / zero are applied to sums there, which for a unit vector is the
 * single product of the defining formula).  Uses the model's scratch: must not overlap a decode
 * step.  FF_ERR_ARG for a batch the path does not serve (or above the model's max_batch). */
int ff_debug_gemv(ff_model *m, int32_t layer, int32_t which, const float *in_dev, float *out_dev,
                  int32_t batch, int32_t path, void *stream);

/* Profiling aid: when buf_dev is non-NULL, every following fused step writes 100 MHz wall-clock
 * stamps into it; NULL switches it off.  With P = 4*n_layers+1 projection phases and W workgroups
 * (see ff_fused_schedule) the buffer must hold 12*P + 72*W uint64:
 *   [0, 12P)          workgroup 0: 12 slots per phase (0 input staged, 1 projection done, 2 first
 *                     tiles requested, 3 staging starts, 6/7 attention start/end)
 *   [12P, 12P+32W)    layer 1, 8 per wave: projection end of QKV/O/GU/DOWN, then their starts
 *   [12P+32W, +40W)   layer 1, per workgroup: 8 per projection (input staging entered, first load
 *                     checked, last light wait done, all fresh, staged, number of stale passes),
 *                     then 8 about its attention work (start, queries seen, rows done, partial
 *                     stored, split maxima seen and merged output stored if it merges, end) */
int ff_debug_timeline(ff_model *m, void *buf_dev);

/* Measurement aid: one launch that reads `bytes` of buf_dev once with the access pattern of the
 * decode kernels' weight stream (n_workgroups workgroups of 256 threads, one contiguous slab each,
 * eight 16-byte non-temporal loads in flight per lane).  Timed by the benchmark to report the
 * streaming-read ceiling of the machine beside the nominal HBM peak. */
int ff_debug_stream_read(const void *buf_dev, size_t bytes, int32_t n_workgroups, void *stream);

/* Ablation of the paper's preliminary study (Section 3, stacked square linear layers on one input
 * vector): y = W[n_layers-1] ... W[1] W[0] x with W bf16 [n_layers][d][d] (row-major [out][in]), x and y
 * fp32 [d] device vectors.  mode 0: one streaming-GEMV launch per layer ("Baseline"); mode 1: one
 * persistent kernel with a tagged hand-over between layers ("Fused"); mode 2: the same with each
 * layer's first weight tiles requested before its input is waited for ("+ Overlap").  d must be a
 * multiple of 2048 in [2048, 32768]; scratch_dev: 2 * align256(4 d) + 256 bytes, 256-byte aligned.
 * The word at scratch offset 2 * align256(4 d) is a status word (0 = ok) that the caller clears. */
int ff_debug_stack_linear(const void *w_dev, int32_t d, int32_t n_layers, const float *x_dev, float *y_dev,
                          int32_t mode, void *scratch_dev, size_t scratch_bytes, void *stream);

/* Ablation switch (the "Fused" vs "+ Overlap" columns of the paper's latency tables, Sections 3 and
 * 5.3): overlap = 0 makes the fused kernel request a projection's first weight tiles only after its
 * input has arrived (no cross-layer memory overlap); nonzero restores the default.  bf16 models with
 * max_batch 1 only (FF_ERR_UNSUPPORTED otherwise).  Results are identical either way. */
int ff_debug_set_overlap(ff_model *m, int32_t overlap);

/* Measurement switch for the attention work list.  By default the fused kernel rebuilds the list
 * every step from the sequences' lengths: each (sequence, kv head) gets one workgroup, the rest of
 * the grid is dealt out in proportion to the rows each sequence has to read, so a ragged batch is
 * cut into slices of about equal length (the paper's Section 6 names load balance at variable
 * context as the case for scheduling at run time; here the list is recomputed per step on the
 * device, its entries keep fixed owners).  by_length = 0 gives every sequence the same number of
 * workgroups, as the paper's static partition does; nonzero restores the default.  Results agree
 * to rounding either way (the slices differ); batches of equal lengths are sliced identically. */
int ff_debug_set_attention_balance(ff_model *m, int32_t by_length);

/* Test hook for the FF_ERR_TIMEOUT path: while `workgroup` is >= 0, that workgroup of every
 * following fused step leaves at once without publishing anything, so each workgroup that needs its
 * output gives up after its own bounded wait (a fraction of a second), all kernels end normally and
 * ff_status reports FF_ERR_TIMEOUT; -1 switches the hook off.  The model must then be created
 * again (see ff_status). */
int ff_debug_mute_workgroup(ff_model *m, int32_t workgroup);

/* Number of device-wide barriers one fused step executes (0: phases are ordered by tagged dataflow;
 * kept for tests of the schedule), and the number of
 * workgroups / threads per workgroup the fused kernel launches with. */
int ff_fused_schedule(const ff_model *m, int32_t *barriers_per_step, int32_t *n_workgroups,
                      int32_t *threads_per_workgroup);

#ifdef __cplusplus
}
#endif
#endif /* FLASHFORMER_H */
