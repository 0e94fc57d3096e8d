/*
 * l2pd.h -- C ABI of the Learn2PD decoding loop for AMD MI355X (gfx950).
 *
 * The library runs the semi-autoregressive masked-diffusion decoding loop of
 * "Learning to Parallel" (arXiv 2509.25188): per denoising step one full
 * bidirectional transformer forward (the paper's mask predictor M(X)), the
 * greedy estimate and confidence of the active block (Eq. 3, Eq. 4), the
 * learned filter f_theta on the block's confidences (Sec. 3.2), the unmask
 * update (Alg. 2) and End-of-Text Prediction (Sec. 3.3, Alg. 3 in App. A);
 * and the training side of the method: the Extremely Greedy Parallel rollout
 * that labels confidences (Sec. 3.1.3, Alg. 1) and the fit of the filter to
 * those labels (Eq. 6, AdamW as in Sec. 4.1).
 *
 * Conventions for every entry point
 *   - Pointers named *_dev are device (HBM) memory owned by the caller; the
 *     library never frees or reallocates them.  Pointers without that suffix
 *     are host memory, read during the call only.
 *   - `stream` is a hipStream_t passed as void*.  Kernels are enqueued on it;
 *     outputs are valid once the caller has synchronised the stream.
 *   - Return value: L2PD_OK (0) or a negative l2pd_status.  Argument checks
 *     happen on the host before anything is launched.  Nothing throws or aborts.
 *   - A context serves one call at a time (its workspace is shared state).
 *   - Weight matrices are row-major [out_features, in_features]; their element
 *     type is desc.dtype (fp32 or bf16).  Norm gains have the same type.
 *   - Token ids are int32.  Sequences of a batch are stored [B, T] row-major,
 *     T = prompt_len + gen_len.
 */
#ifndef L2PD_H
#define L2PD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  L2PD_OK = 0,
  L2PD_EINVAL = -1,   /* bad argument (NULL pointer, inconsistent sizes, NaN threshold, ...) */
  L2PD_ENOMEM = -2,   /* workspace too small (l2pd_filter_train_static: filter beyond the static scratch) */
  L2PD_EHIP = -3,     /* a HIP runtime call failed */
  L2PD_ENOTIMPL = -4  /* shape outside what the kernels support, or a combination of modes that is not built */
} l2pd_status;

enum { L2PD_FP32 = 0, L2PD_BF16 = 1 };

/* Shape of the mask predictor.  The paper uses LLaDA-8B as a black box; this is the LLaDA-style
 * family: pre-norm blocks, RMSNorm, rotary embedding (rotate-half pairing, angle
 * pos * rope_base^(-2i/head_dim)), bidirectional attention, SwiGLU FFN, untied LM head, no biases.
 * bf16 models need d_model and d_ffn multiples of 64 and head_dim 64 or 128. */
typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
  int32_t mask_id, eos_id;      /* ids of [MASK] and of the end-of-text token, both in [0, vocab) */
  float rope_base, rms_eps;
  int32_t dtype;                /* L2PD_FP32 or L2PD_BF16: storage type of all weights */
} l2pd_model_desc;

/* Device pointers to the weights.  The per-layer members are HOST arrays of n_layers device
 * pointers.  The library copies the pointer values at l2pd_create and reads the weights in place. */
typedef struct {
  const void* tok_emb_dev;          /* [vocab, d_model] */
  const void* lm_head_dev;          /* [vocab, d_model] */
  const void* final_norm_g_dev;     /* [d_model] */
  const void* const* attn_norm_g;   /* each [d_model] */
  const void* const* wq;            /* each [d_model, d_model] */
  const void* const* wk;
  const void* const* wv;
  const void* const* wo;
  const void* const* ffn_norm_g;    /* each [d_model] */
  const void* const* w_gate;        /* each [d_ffn, d_model] */
  const void* const* w_up;          /* each [d_ffn, d_model] */
  const void* const* w_down;        /* each [d_model, d_ffn] */
} l2pd_weights;

/* The filter f_theta (Sec. 3.2; Sec. 4.1 "two-layer MLP"): an MLP on c, the block's confidence
 * vector, with ReLU between its layers and a sigmoid on its output.  n_layers = 2 is the paper's filter,
 * p = sigmoid(W2 relu(W1 c + b1) + b2); 1 (p = sigmoid(W1 c + b1)) and 4 are the variants of Table 3,
 * any depth up to L2PD_FILTER_MAX_LAYERS is taken.  Layer k (0-based) maps width in_k to out_k, where
 * in_0 = out_{n_layers-1} = in_dim and every other width is `hidden`.  All fp32, device memory.
 * in_dim must equal block_len. */
#define L2PD_FILTER_MAX_LAYERS 4
typedef struct {
  int32_t n_layers;                               /* 1 .. L2PD_FILTER_MAX_LAYERS */
  int32_t in_dim, hidden;                         /* hidden <= 1024; unused when n_layers == 1 */
  const float* w_dev[L2PD_FILTER_MAX_LAYERS];     /* layer k: [out_k, in_k] row-major */
  const float* b_dev[L2PD_FILTER_MAX_LAYERS];     /* layer k: [out_k] */
} l2pd_filter;

/* Workload hook: add `value` to the logit of `token_id` at generation positions >= gen_pos_from
 * (position 0 = first generated token).  value == 0 disables it. */
typedef struct {
  int32_t token_id, gen_pos_from;
  float value;
} l2pd_logit_bias;

/* KV-cache variants of Sec. 4.3 / Table 2; the paper names them and cites their source, the
 * mechanisms are that source's.  Both keep per-layer K (rotated) and V, rebuilt at every block start,
 * and run the steps of a block on the block's rows only.
 *   PREFIX: the store holds prompt + finished blocks, computed from a forward over that prefix alone;
 *           a step attends to the stored prefix and to the block itself, not to later positions.
 *   DUAL:   the store holds every position, computed from a full bidirectional forward over the
 *           current sequence; a step attends to all positions, the block's own K/V fresh, the rest
 *           (before and after the block) as stored at the block start. */
enum { L2PD_CACHE_NONE = 0, L2PD_CACHE_PREFIX = 1, L2PD_CACHE_DUAL = 2 };

/* End-of-Text Prediction.
 *   BLOCK (Alg. 3): after a block's loop ends, stop if the response holds eos_id.
 *   STEP (Sec. 3.3, the text): after every step, everything after the first eos_id of the response is
 *     discarded and the next step runs on the shortened sequence; block positions after it are never
 *     decoded (they enter the filter as 1.0) and come back as mask_id; decoded_len counts the response
 *     up to and including eos_id.  Full recompute only (kv_cache must be L2PD_CACHE_NONE); the host
 *     waits for the stream after every step, because the length sizes the next launches. */
enum { L2PD_EOTP_OFF = 0, L2PD_EOTP_BLOCK = 1, L2PD_EOTP_STEP = 2 };

/* Batches whose sequences finish blocks (or the decode) at different steps.  The paper decodes one
 * sequence at a time; these are scheduling choices of a batched decoder and change no token.
 *   L2PD_RAGGED_OFF     lock step: every sequence works on the smallest unfinished block index, one that is
 *                       ahead idles until the others reach it.
 *   L2PD_RAGGED_BLOCKS  every sequence works on its own block: same tokens and per-sequence step counts,
 *                       fewer forwards.
 *   L2PD_RAGGED_COMPACT as BLOCKS, and l2pd_generate moves the sequences that are still decoding to the
 *                       leading rows whenever some have finished, so later forwards run over fewer rows
 *                       (with a K/V cache their slices of the stores move with them); l2pd_denoise_step and
 *                       l2pd_generate with L2PD_EOTP_STEP treat it as BLOCKS.
 * With a K/V cache (Sec. 4.3) and per-sequence blocks every sequence's slice of the stores is rebuilt when
 * that sequence enters a new block (a forward over that sequence alone), and a step's block rows sit at
 * per-sequence positions; l2pd_generate then looks at the device state before every step. */
enum { L2PD_RAGGED_OFF = 0, L2PD_RAGGED_BLOCKS = 1, L2PD_RAGGED_COMPACT = 2 };

/* Decode arguments of Alg. 2 / Alg. 3: generation length L_gen, block size s, threshold tau. */
typedef struct {
  int32_t gen_len, block_len;       /* gen_len % block_len == 0, block_len <= 256 */
  float threshold;                  /* unmask position j when p_j > threshold (strict) */
  int32_t eotp;                     /* L2PD_EOTP_OFF, L2PD_EOTP_BLOCK or L2PD_EOTP_STEP */
  int32_t kv_cache;                 /* L2PD_CACHE_NONE, L2PD_CACHE_PREFIX or L2PD_CACHE_DUAL (Sec. 4.3, Table 2);
                                       the cached modes need a context created with use_kv_cache */
  int32_t keep_kv;                  /* l2pd_denoise_step in a cached mode: 0 rebuilds the K/V store from the
                                       tokens first; 1 uses the store as the previous call left it (stepping
                                       through a block after a call that rebuilt it).  l2pd_generate ignores it. */
  int32_t ragged;                   /* L2PD_RAGGED_OFF, L2PD_RAGGED_BLOCKS or L2PD_RAGGED_COMPACT */
  l2pd_logit_bias bias;
} l2pd_decode_cfg;

typedef struct l2pd_ctx l2pd_ctx;

/* Bytes of device workspace a context needs for batches <= max_batch and sequences <= max_seq
 * tokens (prompt + generation).  Returns 0 if the description is invalid. */
size_t l2pd_workspace_bytes(const l2pd_model_desc* desc, int32_t max_batch, int32_t max_seq,
                            int32_t use_kv_cache);

/* Creates a context.  workspace_dev must stay valid and untouched by the caller until
 * l2pd_destroy.  Host-only work: device-side tables are built by the first call that gets a stream. */
int32_t l2pd_create(const l2pd_model_desc* desc, const l2pd_weights* weights, int32_t max_batch,
                    int32_t max_seq, int32_t use_kv_cache, void* workspace_dev,
                    size_t workspace_bytes, l2pd_ctx** out);
void l2pd_destroy(l2pd_ctx* ctx);

/* M(X): one full bidirectional forward over tokens_dev [B, T]; writes the fp32 logits of positions
 * row_begin .. row_begin+row_count-1 of every sequence to logits_out_dev [B, row_count, vocab].
 * (Alg. 2, "conf, pre = M(X)", before the reduction over the vocabulary.) */
int32_t l2pd_forward(l2pd_ctx* ctx, const int32_t* tokens_dev, int32_t B, int32_t T,
                     int32_t row_begin, int32_t row_count, float* logits_out_dev, void* stream);

/* One pass of the while-loop body of Alg. 2 for every sequence of the batch, on device:
 * forward, confidence / greedy token of the active block (Eq. 3, Eq. 4; the mask id is excluded from
 * the vocabulary, ties go to the lowest id), filter, unmask where p_j > threshold plus the masked
 * position of highest confidence, block advance, EoTP check (Alg. 3) when the block completes.
 *
 * tokens_dev [B, prompt_len + gen_len] and state_dev [B, 3] = (block_idx, steps, done) are updated
 * in place.  By default the batch advances in lock step: the active block is the smallest block_idx among
 * sequences that are not done; a sequence that has finished that block idles (state unchanged).  With
 * cfg.ragged every sequence that is not done works on its own block_idx.
 * Optional taps (NULL to skip), all for the active block, written before the update:
 *   logits_dev [B, s, vocab] fp32 (bias applied), conf_dev [B, s], pred_dev [B, s],
 *   filt_dev [B, s] (filter output p), unmask_dev [B, s] (1 where unmasked by this step).
 * With a cached mode in cfg.kv_cache the call first reads state_dev back (it synchronises the
 * stream) and, unless cfg.keep_kv is set, rebuilds the K/V store for the active block from the
 * tokens as they are.
 * In full recompute with L2PD_EOTP_OFF or L2PD_EOTP_BLOCK the call only enqueues kernels (no host
 * synchronisation, no copies, no memset nodes), so after one eager call on a context it may be
 * captured into a HIP graph and replayed: every replay is the next step on the same buffers. */
int32_t l2pd_denoise_step(l2pd_ctx* ctx, int32_t* tokens_dev, int32_t B, int32_t prompt_len,
                          const l2pd_decode_cfg* cfg, const l2pd_filter* filter, int32_t* state_dev,
                          float* logits_dev, float* conf_dev, int32_t* pred_dev, float* filt_dev,
                          uint8_t* unmask_dev, void* stream);

/* Alg. 2 / Alg. 3 for a batch of prompts [B, P].  Outputs:
 *   tokens_out_dev [B, gen_len]: the response slice X[P : P+gen_len]; positions never decoded
 *     because of an EoTP stop still hold mask_id;
 *   steps_out_dev [B]: forwards in which the sequence still had a masked position in its active block;
 *   decoded_len_out_dev [B]: (index of the last decoded block + 1) * block_len; with L2PD_EOTP_STEP the
 *     length of the response up to and including the first eos_id (gen_len if there is none).
 * The step loop, the block pointer and the stop flag live on the device; the host enqueues steps in
 * small chunks and polls a flag between chunks, so the call returns when the last chunk is enqueued. */
int32_t l2pd_generate(l2pd_ctx* ctx, const int32_t* prompt_dev, int32_t B, int32_t P,
                      const l2pd_decode_cfg* cfg, const l2pd_filter* filter, int32_t* tokens_out_dev,
                      int32_t* steps_out_dev, int32_t* decoded_len_out_dev, void* stream);

/* Extremely Greedy Parallel rollout (Sec. 3.1.3; Alg. 1 without its update line): decodes the prompts
 * [B, P] with the rule "unmask position j exactly when the greedy prediction equals the reference answer"
 * reference_dev [B, gen_len], and records one training row per sequence and step:
 *   conf_rows_dev  [B, gen_len, s] fp32: the block's confidences as the filter sees them (1.0 at committed
 *                  positions); row index = step index of that sequence;
 *   label_rows_dev [B, gen_len, s] fp32: 1 where the position may be unmasked (committed, or prediction ==
 *                  reference), else 0;
 *   steps_out_dev  [B]: rows written per sequence (rows beyond stay untouched).
 * When no masked position agrees with the reference, the most confident masked one takes the reference
 * token (label 0), so the rollout ends with X == reference.  Full recompute, no EoTP (cfg.kv_cache and
 * cfg.eotp must be 0; cfg.threshold is ignored); the batch advances in lock step as in l2pd_generate. */
int32_t l2pd_egp_rollout(l2pd_ctx* ctx, const int32_t* prompt_dev, const int32_t* reference_dev, int32_t B,
                         int32_t P, const l2pd_decode_cfg* cfg, float* conf_rows_dev, float* label_rows_dev,
                         int32_t* steps_out_dev, void* stream);

/* Filter training (Sec. 3.2, Eq. 6; Sec. 4.1 names AdamW, learning rate 1e-3, 5,000 epochs): `epochs`
 * full-batch AdamW steps (decoupled weight decay, bias-corrected moments) on the mean binary cross-entropy
 * of sigmoid(f(conf_row)) against label_row over all n_rows * in_dim entries.  The filter's parameters are
 * UPDATED IN PLACE through the pointers of `filter` (device memory, fp32).  opt_state_dev: 2 * n_params
 * floats of device scratch (n_params = sum over the layers of out_k * in_k + out_k; layer after layer,
 * weights before biases), zeroed by the call;
 * loss_out_dev [epochs] (optional) receives the loss of every epoch before its update.  Runs as one
 * workgroup; returns L2PD_ENOTIMPL for filters too large for it (more than 20480 parameters). */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
  int32_t epochs;
} l2pd_train_cfg;
int32_t l2pd_filter_train(const l2pd_filter* filter, const float* conf_rows_dev, const float* label_rows_dev,
                          int64_t n_rows, const l2pd_train_cfg* train_cfg, float* opt_state_dev,
                          float* loss_out_dev, void* stream);

/* l2pd_filter_train for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same training, with the optimiser moments kept in a
 * device array that is part of the library image instead of opt_state_dev.  The call allocates and frees
 * nothing, on the device or through any library.
 *   - Limit: filters of at most 20480 parameters (160 KB of moments per GPU, resident until the process
 *     ends); a larger filter returns L2PD_ENOMEM before anything is launched.  Every other argument and
 *     every result is as for l2pd_filter_train (same kernel, bit-identical parameters and losses).
 *   - The first call on a device looks the array's address up once (HIP loads the library's code object then
 *     if nothing has yet): make one call outside a capture before capturing.
 *   - All calls on one GPU share that GPU's array.  The kernel zeroes the moments before its first epoch, so
 *     nothing survives from call to call; calls that overlap on one GPU (different streams) race. */
int32_t l2pd_filter_train_static(const l2pd_filter* filter, const float* conf_rows_dev,
                                 const float* label_rows_dev, int64_t n_rows, const l2pd_train_cfg* train_cfg,
                                 float* loss_out_dev, void* stream);

/* Timing aid: kernel classes whose launches can be bracketed with HIP events on the launch stream. */
enum {
  L2PD_K_NONE = 0, L2PD_K_GEMM_QKV = 1, L2PD_K_GEMM_O = 2, L2PD_K_GEMM_GATEUP = 3,
  L2PD_K_GEMM_DOWN = 4, L2PD_K_ATTN = 5, L2PD_K_LMHEAD = 6, L2PD_K_NORM = 7, L2PD_K_UPDATE = 8
};
/* Selects one kernel class (L2PD_K_NONE switches timing off) and clears the counters. */
int32_t l2pd_profile_select(l2pd_ctx* ctx, int32_t kernel_class);
/* Synchronises the recorded events and returns the number of timed launches of the selected class
 * since the last select and the sum of their event-pair durations in milliseconds (each includes the gap
 * between the event and the kernel on the stream: an upper bound of the kernel's own time by a few percent). */
int32_t l2pd_profile_read(l2pd_ctx* ctx, int64_t* launches_out, double* total_ms_out);

/* What the last l2pd_generate on this context enqueued (host-side counters, no synchronisation): the number
 * of step launches, and the sum over them of the sequences each ran over (batch size x steps in lock step;
 * less with L2PD_RAGGED_COMPACT once sequences have finished: Sec. 3.3's saving carried over to a batch).
 * Either pointer may be null. */
int32_t l2pd_generate_stats(const l2pd_ctx* ctx, int64_t* steps_out, int64_t* sequence_steps_out);

const char* l2pd_strerror(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* L2PD_H */
