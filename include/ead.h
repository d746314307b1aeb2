/*
 * ead.h -- C ABI of the Entropy Adaptive Decoding library for AMD MI355X (gfx950).
 *
 * Entropy Adaptive Decoding (Section 3 of the paper) generates text with a pair of
 * decoder-only language models that share one vocabulary, a small one M_S and a
 * large one M_L.  After every generated token the Shannon entropy H_t of the
 * active model's next-token distribution (Eq. 1-2, taken on the raw logits) is
 * pushed into a rolling window of w entries; the window mean (Eq. 3) is compared
 * with a threshold tau, and the active model changes when the mean crosses tau
 * and the current model has produced at least d_min tokens (Eq. 4, Algorithm 1).
 *
 * Conventions
 *  - Plain C11.  Every function returns an ead_status; nothing throws or aborts.
 *  - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *    memory on the GPU that was current when the handle was created.
 *  - Weights are BORROWED only for the duration of ead_create(): the library
 *    copies them into its own streaming layout, after which the caller may free
 *    them.  Until the caller does, device memory holds every matrix twice (the
 *    caller's tensors and the library's tiles): about 58 GB for a 0.5 B + 14 B
 *    parameter pair in bf16, half of that afterwards.  Everything else the
 *    library needs (KV caches, gate state, scratch) it allocates in ead_create()
 *    and frees in ead_destroy().
 *  - Precision of a bf16 model: the matrices of the linear layers are kept as IEEE
 *    half, which holds every bf16 value of magnitude 2^-24 .. 65504 exactly (smaller
 *    ones round to a multiple of 2^-24); passes of three or more rows round their
 *    activations to half as well (11 significant bits; values beyond +-65504
 *    saturate) and accumulate in float32; passes of one or two rows keep float32
 *    activations.  K and V are cached in bf16.  Embeddings, gains, the residual
 *    stream, soft-max statistics and the entropy are float32 throughout.
 *  - Outputs are caller-owned host buffers unless the name ends in _dev.
 *  - A handle serves one call at a time (calls are not re-entrant).  Work is
 *    queued on ead_params.hip_stream and every call returns after its results
 *    have reached the host buffers.
 *  - Decoding is greedy by default (token = arg max of the raw logits, lowest
 *    index on a tie); ead_set_sampling() turns on Algorithm 1's sampling step
 *    y ~ softmax(l / T).
 *  - Models: pre-norm decoders with RMSNorm, rotary position embedding
 *    ("rotate-half" pairing, angle pos * theta^(-2i/head_dim)), grouped-query
 *    attention (query head h reads KV head h / (n_heads / n_kv_heads)) and a
 *    SwiGLU feed-forward block; no biases.
 *  - Shape limits: d_model, d_ffn and n_heads*head_dim multiples of 32, at most
 *    15360 (float32 weights: at most 4096); vocab a multiple of 16; head_dim one
 *    of 32, 64, 128; n_heads / n_kv_heads an integer between 1 and 8.
 */
#ifndef EAD_H
#define EAD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EAD_OK = 0,
    EAD_ERR_INVALID_ARG = 1,    /* null pointer, negative size, w < 1, d_min < 1, NaN tau ... */
    EAD_ERR_SHAPE = 2,          /* model shape outside the limits above */
    EAD_ERR_VOCAB_MISMATCH = 3, /* the two models do not share one vocabulary size */
    EAD_ERR_OOM = 4,            /* device or host allocation failed */
    EAD_ERR_SEQ_OVERFLOW = 5,   /* prompt + new tokens exceed max_seq, or batch > max_batch */
    EAD_ERR_NONFINITE = 6,      /* an entropy came out NaN/Inf (non-finite logits) */
    EAD_ERR_DEVICE = 7,         /* a HIP call failed; see ead_last_error() */
    EAD_ERR_NO_DEVICE = 8,      /* no usable GPU */
    EAD_ERR_STATE = 9           /* call order violated (e.g. ead_decode before ead_begin) */
} ead_status;

typedef enum { EAD_F32 = 0, EAD_BF16 = 1 } ead_dtype;
typedef enum { EAD_MODEL_SMALL = 0, EAD_MODEL_LARGE = 1 } ead_model_id;
typedef enum { EAD_NATS = 0, EAD_BITS = 1 } ead_unit;   /* Eq. 2 is written in bits */

/* One decoder.  All pointers are DEVICE pointers; matrices are row-major
 * [out_features, in_features] in `dtype`; the norm gains are always float32. */
typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rms_eps, rope_theta;
    int32_t dtype;                       /* ead_dtype of the matrices */
    const void *embed;                   /* [vocab, d_model]                      */
    const void *const *wq;               /* host array of n_layers device pointers, each [n_heads*head_dim, d_model] */
    const void *const *wk;               /* ... each [n_kv_heads*head_dim, d_model] */
    const void *const *wv;               /* ... each [n_kv_heads*head_dim, d_model] */
    const void *const *wo;               /* ... each [d_model, n_heads*head_dim]    */
    const void *const *w_gate;           /* ... each [d_ffn, d_model]               */
    const void *const *w_up;             /* ... each [d_ffn, d_model]               */
    const void *const *w_down;           /* ... each [d_model, d_ffn]               */
    const float *const *norm_attn;       /* ... each [d_model] float32              */
    const float *const *norm_ffn;        /* ... each [d_model] float32              */
    const float *norm_final;             /* [d_model] float32                       */
    const void *lm_head;                 /* [vocab, d_model]                        */
} ead_model_desc;

/* Inputs of Algorithm 1 other than the prompt and the models. */
typedef struct {
    int32_t window;        /* w >= 1; the paper's experiments use 5                         */
    float tau;             /* threshold on the window mean, in `unit`                        */
    int32_t d_min;         /* minimum tokens by one model before a switch, >= 1; paper: 10   */
    int32_t unit;          /* ead_unit of tau and of every reported entropy                  */
    int32_t max_batch;     /* sequences decoded together, >= 1                               */
    int32_t max_seq;       /* prompt + generated tokens per sequence                         */
    int32_t eos_id;        /* stop a sequence after this token; -1 = never                   */
    void *hip_stream;      /* hipStream_t to queue work on (borrowed); NULL = default stream */
} ead_params;

typedef struct ead_handle ead_handle;

/* Counters since ead_begin() (or the last ead_reset_stats()). */
typedef struct {
    int64_t tokens_small, tokens_large;    /* generated tokens by model                      */
    int64_t switches;                      /* model changes summed over sequences            */
    int64_t steps_small, steps_large;      /* forward passes that emitted tokens             */
    int64_t catchup_rows_small, catchup_rows_large; /* extra positions a model had to consume
                                              because the other model had produced them      */
    int64_t host_syncs;                    /* times the host waited for a gate decision      */
    double algorithmic_bytes;              /* weights streamed + KV read, by the byte model:
                                              per pass, the model's weight bytes plus, per
                                              token row, kv_bytes_per_position * keys read   */
    double large_share;                    /* tokens_large / (tokens_small + tokens_large)   */
    double param_ratio;                    /* Table 1 footnote: (a*P_S + b*P_L) / P_L        */
} ead_stats;

/* ---- life cycle ---------------------------------------------------------------- */

/* Build a handle for a model pair (Algorithm 1's M_S, M_L, tau, w, d_min).
 * Copies both models into the library's layout and allocates KV caches for
 * max_batch x max_seq positions per model (max_seq rounded up to a multiple of
 * 32 internally; in the weight dtype; bf16 models keep V a second time,
 * transposed, for the matrix-core attention: 1.5 x the K + V bytes in all).
 * Errors: INVALID_ARG, SHAPE,
 * VOCAB_MISMATCH, OOM, NO_DEVICE, DEVICE.  *out is NULL on error. */
ead_status ead_create(const ead_model_desc *small_model, const ead_model_desc *large_model,
                      const ead_params *params, ead_handle **out);
void ead_destroy(ead_handle *h);
/* Message of the last failed call on this handle (handle-owned string); with
 * h == NULL, the message of the last failed ead_create() on this thread. */
const char *ead_last_error(const ead_handle *h);
/* Change tau / d_min / window / unit / eos_id between runs (max_* and the stream stay). */
ead_status ead_set_gate(ead_handle *h, int32_t window, float tau, int32_t d_min, int32_t unit,
                        int32_t eos_id);

/* ---- Algorithm 1 --------------------------------------------------------------- */

/* Whole algorithm for `batch` independent sequences (each row is its own instance
 * of Algorithm 1: own window, counter and current model).
 *   prompt_tokens  host, the prompts concatenated, sum(prompt_lens) entries
 *   prompt_lens    host [batch], each >= 1
 *   out_tokens     host [batch, max_new_tokens]   generated tokens y
 *   out_model_id   host [batch, max_new_tokens]   model that produced each token (0 = M_S)
 *   out_entropy    host [batch, max_new_tokens]   H_t of the logits the token came from
 *   out_window_mean host [batch, max_new_tokens]  window mean after H_t (nullable)
 *   out_lens       host [batch]                   tokens generated per row (eos may cut it)
 * Equivalent to ead_begin + ead_decode(max_new_tokens) + ead_fetch. */
ead_status ead_generate(ead_handle *h, const int32_t *prompt_tokens, const int32_t *prompt_lens,
                        int32_t batch, int32_t max_new_tokens, int32_t *out_tokens,
                        uint8_t *out_model_id, float *out_entropy, float *out_window_mean,
                        int32_t *out_lens);

/* Start a run: reset all state, load the prompts, and let BOTH models consume
 * every prompt token but the last (so that no entropy is recorded yet and the
 * first decode step produces the first token).  max_new_tokens bounds the run. */
ead_status ead_begin(ead_handle *h, const int32_t *prompt_tokens, const int32_t *prompt_lens,
                     int32_t batch, int32_t max_new_tokens);
/* Start the run over from the state ead_begin() left: Algorithm 1's initialisation (empty
 * window, M = M_S, c = 0, nothing generated) with both models still holding the prompts of the
 * last ead_begin() in their caches, so no prompt pass is repeated.  Takes the gate, forced-model,
 * schedule and sampling settings in force now; max_new_tokens bounds the new run.
 * Errors: STATE when the caches no longer hold those prompts (no ead_begin yet, or an
 * ead_score / ead_replay since), SEQ_OVERFLOW, INVALID_ARG. */
ead_status ead_rewind(ead_handle *h, int32_t max_new_tokens);
/* Run n_steps iterations of Algorithm 1's loop for every unfinished row
 * (one token per row per step, including any catch-up the active model needs).
 * Returns after the last step's work has finished on the GPU. */
ead_status ead_decode(ead_handle *h, int32_t n_steps);
/* Free-running batch: rows are independent instances of Algorithm 1, so nothing forces them to move in
 * steps.  Runs the grouped schedule (see ead_set_schedule; its start / stop fractions apply) until the batch
 * as a whole has produced at least n_tokens more tokens, every row free to go on as far as max_lead tokens
 * ahead of the unfinished row that has produced the fewest (and never past the run's max_new_tokens).  No new
 * forward pass is started once the count is reached; passes in flight finish, so a few more tokens than
 * asked for may come out (ead_get_stats counts them).  Per row the tokens are those ead_decode would have
 * produced (up to the rounding differences between passes of different width).  Batches of up to 512. */
ead_status ead_decode_tokens(ead_handle *h, int64_t n_tokens, int32_t max_lead);
/* Copy what has been generated so far to host buffers laid out as in
 * ead_generate with row stride `stride` (>= tokens generated). Any pointer may be NULL. */
ead_status ead_fetch(ead_handle *h, int32_t stride, int32_t *out_tokens, uint8_t *out_model_id,
                     float *out_entropy, float *out_window_mean, int32_t *out_lens);

/* ---- teacher-forced entry points (parity tests) --------------------------------- */

/* One model over one token sequence: logits, entropy and arg max at every
 * position (position i predicts token i+1).
 *   tokens host [len]; out_logits host [len, vocab] float32 (nullable);
 *   out_entropy host [len] (nullable); out_argmax host [len] (nullable). */
ead_status ead_score(ead_handle *h, int32_t which_model, const int32_t *tokens, int32_t len,
                     float *out_logits, float *out_entropy, int32_t *out_argmax);

/* Algorithm 1 along a GIVEN trajectory: at generated position i the logits come
 * from model forced_model_id[row, i] (with whatever catch-up that model needs), the
 * token appended is forced_tokens[row, i], and the library reports what it computed:
 *   out_argmax [batch, n_new]: the token the library itself would have emitted there (the arg
 *   max, or its sampled token while a temperature is set); out_entropy, out_window_mean as in
 *   ead_generate,
 *   out_decision [batch, n_new]: the model Eq. 4 selects for the next token when the
 *   current model is forced_model_id[row, i] and the dwell counter follows the forced ids.
 * All arrays are host memory; prompts as in ead_generate. */
ead_status ead_replay(ead_handle *h, const int32_t *prompt_tokens, const int32_t *prompt_lens,
                      int32_t batch, int32_t n_new, const int32_t *forced_tokens,
                      const uint8_t *forced_model_id, int32_t *out_argmax, float *out_entropy,
                      float *out_window_mean, uint8_t *out_decision);

/* ---- the entropy / gate epilogue on its own (Eq. 1-4) ---------------------------- */

/* Row-wise entropy (Eq. 1-2) and arg max of a logits matrix already in device memory.
 *   logits_dev [rows, vocab] of `dtype`, row-major; H_dev [rows] float32 in `unit`;
 *   argmax_dev [rows] int32 (nullable).  Asynchronous on `hip_stream`.
 * Limits: 1 <= rows <= 4096, vocab a multiple of 8 and at most 1048576.
 * The per-chunk statistics go through a 6 MB buffer per device that the first call on that
 * device allocates and the process keeps; all calls on a device share it, so calls whose
 * work overlaps on the GPU (different streams) race: issue them on one stream or wait in between. */
ead_status ead_entropy_argmax(const void *logits_dev, int32_t dtype, int32_t rows, int32_t vocab,
                              int32_t unit, float *H_dev, int32_t *argmax_dev, void *hip_stream);
/* The same computation for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid it): this entry point calls no
 * allocation routine at all.  Its per-chunk statistics go to a 384 KB array that is part of
 * the library's device image (one copy per GPU, held until the process ends), which bounds
 * the input: rows * chunks <= 16384, where chunks = the number of pieces a row is cut into
 * (10 at vocab 151936 and 64 rows; at most 64).  Larger inputs are rejected with
 * EAD_ERR_INVALID_ARG and a message that names the limit.  Results are bit-identical to
 * ead_entropy_argmax on the same input.  Every call on a GPU uses that GPU's one array:
 * calls whose work overlaps on the GPU race, as above.  Nothing in it needs clearing
 * between calls (every statistic a call reads it has written itself). */
ead_status ead_entropy_argmax_static(const void *logits_dev, int32_t dtype, int32_t rows, int32_t vocab,
                                     int32_t unit, float *H_dev, int32_t *argmax_dev, void *hip_stream);

/* Rolling window + switch rule (Eq. 3-4) for `rows` independent sequences, state on device
 * (1 <= rows <= 4096).  A gate owns the scratch of its own entropy passes, so gates on
 * different streams do not interfere; one gate serves one call at a time. */
typedef struct ead_gate ead_gate;
ead_status ead_gate_create(int32_t rows, int32_t window, float tau, int32_t d_min, void *hip_stream,
                           ead_gate **out);
/* Feed one entropy per row (H_dev [rows] float32, already in the unit of tau).
 * Writes, all nullable device pointers: model_id_dev [rows] uint8 = model that was
 * current for this token, window_mean_dev [rows] float32, next_model_dev [rows] uint8. */
ead_status ead_gate_step(ead_gate *g, const float *H_dev, uint8_t *model_id_dev,
                         float *window_mean_dev, uint8_t *next_model_dev);
/* Entropy + arg max of logits_dev [rows, vocab] followed by the gate step, in one call. */
ead_status ead_gate_step_logits(ead_gate *g, const void *logits_dev, int32_t dtype, int32_t vocab,
                                int32_t unit, float *H_dev, int32_t *argmax_dev,
                                uint8_t *model_id_dev, float *window_mean_dev,
                                uint8_t *next_model_dev);
/* The same for n_steps consecutive steps without returning to the host: step s reads the
 * tensor logits_dev_list[s % n_tensors] (a HOST array of device pointers, each
 * [rows, vocab] of `dtype`).  Entropies of several steps are computed per launch; the
 * window and the switch rule then take the steps in order.  Outputs (nullable device
 * pointers) are [n_steps, rows]: H_dev, argmax_dev, model_id_dev (model current for that
 * step's token), window_mean_dev.  Asynchronous on the gate's stream. */
ead_status ead_gate_run_logits(ead_gate *g, const void *const *logits_dev_list, int32_t n_tensors,
                               int32_t n_steps, int32_t dtype, int32_t vocab, int32_t unit,
                               float *H_dev, int32_t *argmax_dev, uint8_t *model_id_dev,
                               float *window_mean_dev);
ead_status ead_gate_reset(ead_gate *g);
void ead_gate_destroy(ead_gate *g);

/* ---- bookkeeping ----------------------------------------------------------------- */
ead_status ead_get_stats(ead_handle *h, ead_stats *out);
ead_status ead_reset_stats(ead_handle *h);
/* Run only one model for every row (0 / 1), or follow the gate (-1, the default).
 * Used to time small-only and large-only decoding on the same prompts. */
ead_status ead_force_model(ead_handle *h, int32_t which_model_or_minus1);
/* Algorithm 1's sampling step.  temperature = 0 (default): greedy, the token is the arg max of
 * the raw logits (lowest index on ties).  temperature > 0: the token is drawn from
 * softmax(logits / temperature) inside the LM head's epilogue, as
 * argmax_i (l_i / T + g_i) with g_i = -ln(-ln u_i) (Gumbel-max), u_i from Philox-4x32-10 keyed
 * by `seed` with counter (i / 4, index of the generated token, row of the batch, 0) -- a run
 * is reproducible from (seed, prompts).  Entropies are those of the raw logits either way
 * (Section 3.1).  In ead_replay the forced tokens are followed; the tokens the library
 * would have drawn are what it reports.  Takes effect from the next decode step.  The
 * single-kernel decode path (ead_set_fused) decodes greedily and is not used while
 * temperature > 0. */
ead_status ead_set_sampling(ead_handle *h, float temperature, uint64_t seed);
/* How rows of a batch are stepped.  grouped = 0 (default): lock step, every unfinished row
 * produces one token per step.  grouped = 1: rows are independent instances of Algorithm 1,
 * so rows served by the small model run ahead while rows that switched to the large model
 * wait; the large model starts running when at least start_fraction of the unfinished rows
 * wait for it and keeps running until fewer than stop_fraction do, so its weights are streamed
 * once for many rows.  Outputs per row are the same (up to the rounding differences between
 * passes of different width).  ead_decode(n) then lets every row produce up to n more tokens. */
ead_status ead_set_schedule(ead_handle *h, int32_t grouped, float start_fraction, float stop_fraction);
/* Single-row decode steps can run as ONE persistent kernel per step (grid barriers
 * instead of kernel boundaries, weight prefetch across them) instead of the per-layer
 * kernels that wider batches use.  Off by default (on this hardware the per-layer kernels
 * are the faster of the two); on = 1 selects it for the shapes it is built for (the
 * per-layer kernels are used regardless for any other shape): for bf16 models the variant
 * whose fetching waves stream the weights through a ring in LDS, for float32 models the
 * one that buffers them in registers; on = 2 selects the register-buffered variant for
 * bf16 models as well.  All paths compute the same thing; tests compare them. */
ead_status ead_set_fused(ead_handle *h, int32_t on);

/* Per-kernel timing for roofline reports.  While enabled, every kernel launch of the
 * decode path is bracketed by HIP events on the handle's stream (this slows decoding
 * down: use it on a separate, untimed run).  ead_profile_read() waits for the stream,
 * then returns one entry per kernel kind and model with the summed event time and the
 * algorithmic bytes of those launches (weight bytes of the matrix for linear layers,
 * K/V bytes read for attention, 0 for bookkeeping kernels). */
typedef struct {
    char name[48];          /* e.g. "linear_fma_swiglu/large" */
    int64_t launches;
    double total_ms;
    double bytes;
} ead_kernel_profile;
ead_status ead_profile_enable(ead_handle *h, int32_t on);   /* also clears what was collected */
ead_status ead_profile_read(ead_handle *h, ead_kernel_profile *out, int32_t capacity, int32_t *n_out);
/* Bracket only the launches of one kernel class (a name as ead_profile_read reports it, e.g.
 * "linear_mfma_swiglu/large"), so that timing the kernel a roofline entry is about disturbs the
 * rest of the run as little as possible; NULL or "" = every class again (the default). */
ead_status ead_profile_select(ead_handle *h, const char *name);
/* Library version as major*10000 + minor*100 + patch. */
int32_t ead_version(void);

#ifdef __cplusplus
}
#endif
#endif /* EAD_H */
