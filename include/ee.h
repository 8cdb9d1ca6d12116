/*
 * ee.h -- C ABI of the early-exit decode library for MI355X (gfx950).
 *
 * One autoregressive decode step through a decoder-only transformer with early-exit heads, using
 * KV recomputation (paper: Section 4, paragraph "KV recomputation"; Appendix D.3 "Inference
 * service").  Tokens that leave at an early exit are kept on a per-sequence list of recent tokens
 * whose deep-layer KV is missing; every later step that goes deeper carries them along, so that
 * their KV entries are filled.  A full-depth step is forced when the list reaches max_pending
 * (Appendix D.3, last sentence).  The exit rule is the confidence rule of Section 5.2: at each
 * exit, in depth order, leave if the largest next-token probability reaches the threshold; a
 * threshold of 1 disables the exits.
 *
 * Conventions
 *   - Plain C.  Every call returns 0 (EE_OK) or a negative error code; ee_strerror() names it and
 *     ee_last_hip_error() returns the HIP status behind the last EE_ERR_HIP.
 *   - The library allocates NO device memory.  The caller passes device buffers (sizes come from
 *     the *_bytes queries; every buffer must be 256-byte aligned) and a HIP stream as `void*`
 *     (NULL = the default stream).  Small pinned host buffers are allocated at create time.
 *   - "dev_" arguments are device pointers, everything else is host memory, read or written only
 *     during the call.
 *   - A model is immutable once its tensors are set and may serve several caches.  A cache handle,
 *     and a model while a call is running on it, must not be used from two threads at once.
 *   - All work is enqueued on the given stream; calls that return tokens wait for the head results of
 *     that work before returning (the host needs the exit decision to know which layers to launch
 *     next): the results arrive in pinned host memory that the call polls, written by the last kernel
 *     of the step, so nothing of the step is in flight when it returns.  ee_prefill, ee_kv_cache_flush
 *     and the read-backs synchronise the stream.
 */
#ifndef EE_H
#define EE_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

enum { EE_F32 = 0, EE_BF16 = 1 };

enum {
    EE_OK = 0,
    EE_ERR_CONFIG = -1, /* bad shapes, exits not ascending, unsupported sizes */
    EE_ERR_NOMEM = -2,  /* a caller buffer is too small, or the KV block pool is exhausted */
    EE_ERR_RANGE = -3,  /* token >= vocab, bad sequence id, position beyond max_positions */
    EE_ERR_STATE = -4,  /* tokens / pending_mask disagree with the cache state; missing tensors */
    EE_ERR_IO = -5,     /* weight file unreadable or malformed */
    EE_ERR_HIP = -6,    /* a HIP call failed; see ee_last_hip_error() */
    EE_ERR_ARG = -7     /* NULL or misaligned pointer, bad count */
};

/* Compile-time limits of one launch */
#define EE_MAX_ROWS 256 /* rows (current + deferred tokens of all sequences) in one step */
#define EE_MAX_SEQS 64  /* sequences in one step */
#define EE_MAX_EXITS 8

/*
 * Model: pre-RMSNorm decoder, rotary position embedding (half-split pairs, angle
 * pos * rope_base^(-2i/head_dim)), SwiGLU MLP, no biases.  Exit i sits after layer exit_layers[i]
 * (1-based).  By default (exit_flags = 0) it is an RMSNorm gain plus its own d_model x vocab matrix;
 * exit_flags selects the other structures of Section 2 ("Model architectures": an output embedding
 * matrix, an optional normalisation in front of it, optionally an MLP before that, input and output
 * embeddings tied or untied):
 *   EE_EXIT_NO_NORM    exits apply their output embedding to the residual stream as it is (the final
 *                      head keeps its norm); the model has no EE_T_EXIT_NORM tensors;
 *   EE_TIE_EMBEDDINGS  every exit and the final head use the input embedding matrix; the model has no
 *                      EE_T_EXIT_HEAD / EE_T_FINAL_HEAD tensors (the library keeps the embedding twice:
 *                      by rows for the token look-up, in tile order for the heads);
 *   EE_EXIT_MLP        exit i starts with an MLP block of its own, of the same form as a layer's:
 *                      x' = x + W_d (silu(W_g h) * (W_u h)), h = rmsnorm(x; g_mlp); its (norm and) output
 *                      embedding read x', the backbone's x is unchanged.  Tensors EE_T_EXIT_MLP_NORM,
 *                      EE_T_EXIT_WG, EE_T_EXIT_WU, EE_T_EXIT_WD per exit, hidden width d_ff.
 *   EE_EXIT_LAYER      exit i starts with a complete Transformer layer of its own (Section 2 and Appendix D.1 name it
 *                      next to the MLP), the same block as a backbone layer with the exit's weights, applied to the
 *                      hidden states at the exit's depth: its attention at position t runs over the K and V this
 *                      layer produced at positions 0..t.  Its output feeds the exit's (norm and) output embedding;
 *                      the backbone's x is unchanged.  Every position that passes the exit's depth leaves its K and
 *                      V in that layer, whether or not the exit is evaluated for it (exits disabled, forced step,
 *                      deferred row): the cache holds them as layer n_layers + i, filled together with the segment
 *                      that ends at the exit.  Tensors EE_T_EXIT_ATTN_NORM, EE_T_EXIT_WQ/WK/WV/WO and, for its MLP
 *                      half, EE_T_EXIT_MLP_NORM, EE_T_EXIT_WG/WU/WD.  Not together with EE_EXIT_MLP (EE_ERR_CONFIG);
 *                      ee_prefill_scored does not support it (EE_ERR_CONFIG).
 * Setting a tensor that the configured structure does not have returns EE_ERR_CONFIG.
 * Supported: d_model = n_heads*head_dim; head_dim in {32, 64, 128}; d_model, d_ff multiples of 32;
 * vocab a multiple of 32.
 */
typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ff, vocab;
    int32_t n_exits, exit_layers[EE_MAX_EXITS]; /* ascending, each in [1, n_layers-1] */
    int32_t dtype;                              /* EE_F32 | EE_BF16: storage of matrices, embedding, KV */
    int32_t max_positions;                      /* longest sequence (prompt + generated) */
    float rms_eps, rope_base;
    int32_t exit_flags;                         /* EE_EXIT_NO_NORM | EE_TIE_EMBEDDINGS | EE_EXIT_MLP | EE_EXIT_LAYER; 0 = default */
    /* Tuning, not part of the model (and not stored in weight files); 0 = default for each. */
    int32_t prefill_rows;        /* rows per pass of the prompt-phase GEMM path: 0 = 2048, n > 0 = min(n, 8192) rounded to
                                    128 (at least 128), n < 0 = path off (prompts then go through the decode kernels) */
    int32_t gemm_min_workgroups; /* a decode GEMM over many rows gives a workgroup several 16-column tiles as long as
                                    this many workgroups remain: 0 = 512; tests lower it so that small models reach
                                    those kernel variants */
    int32_t scored_head_terms;   /* bf16 terms of the activations in the heads that ee_prefill_scored evaluates on
                                    every position: 0 or 1 = the leading term only (half the matrix-core work; the
                                    logits then carry the rounding of the head's input to bf16, about 1e-3 of their
                                    largest), 2 = both terms, as everywhere else.  Nothing but pos_token, pos_conf
                                    and pos_nll depends on it: the prompt's own token and exit are decided by the
                                    decode heads on the last row. */
} ee_config;

enum { EE_EXIT_NO_NORM = 1, EE_TIE_EMBEDDINGS = 2, EE_EXIT_MLP = 4, EE_EXIT_LAYER = 8 };

/* Tensor kinds for ee_model_set_tensor (index = layer for per-layer kinds, exit number for EXIT_*). */
enum {
    EE_T_EMBED = 0,      /* [vocab][d_model]                                        */
    EE_T_ATTN_NORM = 1,  /* [d_model] fp32 gain, per layer                          */
    EE_T_WQ = 2,         /* [d_model][d_model], row = output feature (y = W x)      */
    EE_T_WK = 3,
    EE_T_WV = 4,
    EE_T_WO = 5,
    EE_T_MLP_NORM = 6,   /* [d_model] fp32 gain                                     */
    EE_T_WG = 7,         /* [d_ff][d_model]                                         */
    EE_T_WU = 8,         /* [d_ff][d_model]                                         */
    EE_T_WD = 9,         /* [d_model][d_ff]                                         */
    EE_T_EXIT_NORM = 10, /* [d_model] fp32 gain, per exit                           */
    EE_T_EXIT_HEAD = 11, /* [vocab][d_model], per exit                              */
    EE_T_FINAL_NORM = 12,
    EE_T_FINAL_HEAD = 13,
    EE_T_EXIT_MLP_NORM = 14, /* [d_model] fp32 gain, per exit (EE_EXIT_MLP only)    */
    EE_T_EXIT_WG = 15,       /* [d_ff][d_model], per exit                           */
    EE_T_EXIT_WU = 16,       /* [d_ff][d_model]                                     */
    EE_T_EXIT_WD = 17,       /* [d_model][d_ff]                                     */
    EE_T_EXIT_ATTN_NORM = 18, /* [d_model] fp32 gain, per exit (EE_EXIT_LAYER only; 14..17 are that layer's MLP half) */
    EE_T_EXIT_WQ = 19,        /* [d_model][d_model], per exit                        */
    EE_T_EXIT_WK = 20,
    EE_T_EXIT_WV = 21,
    EE_T_EXIT_WO = 22,
    EE_T_KINDS = 23
};

typedef struct ee_model ee_model;
typedef struct ee_kv_cache ee_kv_cache;

const char* ee_strerror(int code);
int ee_last_hip_error(void);

/* ---------------------------------------------------------------- model */

/* Sizes of the two device buffers a model needs.  weight_bytes holds the packed weights and the
 * rotary table; workspace_bytes holds per-step activations for up to max_rows rows
 * (1 <= max_rows <= EE_MAX_ROWS) and max_seqs sequences per step (1 <= max_seqs <= EE_MAX_SEQS). */
int ee_model_bytes(const ee_config* cfg, int max_rows, int max_seqs, size_t* weight_bytes,
                   size_t* workspace_bytes);

/* Creates a model over the caller's device buffers; no tensor is set yet.  Enqueues the rotary table
 * initialisation on `stream`. */
int ee_model_create(const ee_config* cfg, void* dev_weights, size_t weight_bytes, void* dev_workspace,
                    size_t workspace_bytes, int max_rows, int max_seqs, void* stream, ee_model** out);

/* Sets one tensor from a DEVICE array in the plain row-major layout given above (matrices and the
 * embedding in the model's dtype, gains fp32).  The library repacks it into its own layout inside
 * dev_weights (enqueued on `stream`; dev_src may be reused once the stream has passed this point).
 * n_elems must equal the tensor's element count. */
int ee_model_set_tensor(ee_model* m, int kind, int index, const void* dev_src, size_t n_elems, void* stream);

/* Reads a weight file and sets every tensor.  File: the 8 bytes "EEWT0001", the ee_config struct,
 * then every tensor in the order EMBED, per layer {ATTN_NORM, WQ, WK, WV, WO, MLP_NORM, WG, WU, WD},
 * per exit {EXIT_NORM, EXIT_HEAD}, FINAL_NORM, FINAL_HEAD, each as raw little-endian elements.
 * A model with exit_flags != 0 is stored as "EEWT0002": exit_flags follows rope_base in the config, and
 * the per-exit group is {EXIT_ATTN_NORM, EXIT_WQ, EXIT_WK, EXIT_WV, EXIT_WO (with EE_EXIT_LAYER)}, {EXIT_MLP_NORM,
 * EXIT_WG, EXIT_WU, EXIT_WD (with EE_EXIT_MLP or EE_EXIT_LAYER)}, {EXIT_NORM (unless
 * EE_EXIT_NO_NORM)}, {EXIT_HEAD (unless tied)}; FINAL_HEAD is absent when tied.
 * dev_staging is a device scratch buffer of at least staging_bytes = the largest tensor. */
int ee_model_load(const ee_config* cfg, const char* weights_path, void* dev_weights, size_t weight_bytes,
                  void* dev_workspace, size_t workspace_bytes, int max_rows, int max_seqs, void* dev_staging,
                  size_t staging_bytes, void* stream, ee_model** out);

int ee_model_free(ee_model* m);

/* Test hook, host only (no GPU is touched): the step plan that ee_decode_step and ee_kv_cache_flush apply to one
 * sequence (Section 4: the deferred tokens join the current token's pass; Appendix D.3: a full-depth pass is forced
 * once the list has reached the cap).  filled[n_segments] (host, in/out) are the sequence's fill watermarks:
 * filled[s] = positions whose K and V are present in every layer of segment s, non-increasing in s; the
 * deferred tokens are the positions [filled[last], filled[0]).  For a step whose current token sits at
 * `position` (= filled[0]; negative: a flush) the call reports *forced (1 if the list has reached max_pending)
 * and, per segment, the inclusive range of positions row_lo[s]..row_hi[s] that pass through it (refeed != 0:
 * deferred tokens re-enter at layer 1; else they resume where their KV is missing).  If reached >= 0 the
 * watermarks are then advanced as when the step ended in segment `reached` (a flush must reach the last one);
 * reached < 0 leaves them unchanged.  forced, row_lo, row_hi may be NULL.  EE_ERR_STATE if the watermarks are not
 * non-increasing, EE_ERR_ARG on bad counts. */
int ee_debug_plan(int n_segments, int32_t* filled, int position, int max_pending, int refeed, int reached,
                  int32_t* forced, int32_t* row_lo, int32_t* row_hi);
/* Measurement hook: the confidence every head reported in the latest ee_decode_step, conf[n_seqs][n_exits+1] (host;
 * row b = the b-th sequence of that call, column i = exit i, last column = final head); -1 where the head was not
 * evaluated for that sequence in that step (the token had left at a shallower exit, exits disabled or step forced).
 * The benchmark uses it to report the confidence distribution at each exit (Section 5.2: the rule compares exactly
 * this number with the threshold). */
int ee_debug_step_confidences(const ee_model* m, int n_seqs, float* conf);
/* Test hook: if dev_logits != NULL, every head evaluation also stores its fp32 logits there,
 * [row][vocab] for the rows it evaluates (capacity_rows rows).  NULL switches it off. */
int ee_debug_set_logits(ee_model* m, void* dev_logits, int capacity_rows);

/* Measurement hook (used by the benchmark's roofline figure): between begin and end, every launch of
 * one kernel family carries a HIP event pair attached to the dispatch on the launch stream, so each
 * pair measures that kernel's execution time.  end() waits for the recorded events and returns how
 * many launches were timed and their summed duration.  At most max_launches are recorded; later
 * ones run untimed.  (EE_K_ATTN times the main attention kernel, not the split merge after it.) */
enum { EE_K_QKV = 0, EE_K_ATTN = 1, EE_K_OPROJ = 2, EE_K_SWIGLU = 3, EE_K_DOWN = 4, EE_K_HEAD = 5, EE_K_KINDS = 6 };
int ee_profile_begin(ee_model* m, int kernel, int max_launches);
int ee_profile_end(ee_model* m, int32_t* n_launches, float* total_ms);
/* Sampling for the hook above: from the next ee_profile_begin on, only every `every`-th launch (>= 1; 1 = all, the
 * default) of the family carries an event pair.  An event pair costs a launch about 5 us of queue time, which a
 * throughput figure taken in the same region should not pay 32 times a step.  EE_ERR_ARG while a measurement runs. */
int ee_profile_every(ee_model* m, int every);

/* Measurement hook: a kernel that only reads (16 bytes per lane and load, eight loads in flight per wave) is run
 * n_launches times (1..1000) back to back over `bytes` bytes of the model's own weight buffer (0, or more than the
 * buffer holds: all of it; a shorter read moves its start between launches), timed with a HIP event pair on
 * `stream`; *gb_per_s (host) receives bytes read / time in 1e9 bytes per second.  It is what this GPU's memory
 * delivers to a pure read of that size, launch overhead included: the benchmark quotes the decode step against it
 * beside the nominal 8 TB/s (Section 4 relies on weight streaming dominating a decode step).  Blocks until done. */
int ee_measure_stream_read(ee_model* m, size_t bytes, int n_launches, float* gb_per_s, void* stream);

/* Test hook: the kernels reduce over the lanes of a wave (sums of squares, the soft-max maxima and sums of the
 * attention of Section 4's decode step) with lane swaps instead of shuffles through the LDS; this runs both forms on
 * a million pseudo-random values (on the model's workspace, so not while a step is in flight) and stores in
 * *mismatches (host) how many results differ in any bit: 0 is the contract.  Blocks until done. */
int ee_debug_lane_reductions(ee_model* m, int32_t* mismatches, void* stream);

/* ---------------------------------------------------------------- KV cache */

/* How the deferred tokens of this cache are carried along (Section 4, "KV recomputation").  on = 0 (default):
 * each resumes from the residual row saved at the depth it reached and joins only the layers it still lacks.
 * on = 1: the paper's wording taken literally, the deferred tokens are fed again from the embedding, so
 * every layer of the step sees them and rewrites their (identical) shallow KV entries.  Results are the same;
 * the second does more work per step.  The mode can change only while no sequence of the cache has a deferred
 * token (right after creation, a flush or a full-depth step of every sequence): a saved residual row means
 * different things in the two modes.  EE_ERR_STATE otherwise; setting the mode it already has always succeeds. */
int ee_kv_cache_set_refeed(ee_kv_cache* c, int on);
/* KV cache with per-sequence lists of deferred tokens (Section 4, "KV recomputation"; Appendix D.3).
 * The cache is paged: a pool of blocks of block_tokens positions (a multiple of 32), shared by up to
 * max_seqs sequences, max_tokens_total positions in all.  Besides K and V it holds, per sequence, the
 * residual rows of the deferred tokens (max_pending + 1 rows) so that a deferred token resumes above
 * the depth it reached instead of starting again from layer 1 -- the KV entries it produces are the
 * same.
 * max_pending is the cap on a sequence's list of deferred tokens (Appendix D.3: once the list has reached a
 * pre-set length, a full pass is forced): a step that starts with max_pending deferred tokens runs to full depth
 * with the exits switched off.  1..EE_MAX_ROWS-1; <= 0 means no cap: no step is ever forced, the store holds
 * max_rows rows per sequence, and a step whose rows (deferred + current, over all its sequences) exceed the
 * model's max_rows fails with EE_ERR_NOMEM before anything is changed -- ee_kv_cache_flush the sequences and
 * call again.  The same EE_ERR_NOMEM applies with a cap when the batch's lists together outgrow max_rows. */
int ee_kv_cache_bytes(const ee_model* m, int max_seqs, int64_t max_tokens_total, int block_tokens,
                      int max_pending, size_t* bytes);
int ee_kv_cache_create(const ee_model* m, int max_seqs, int64_t max_tokens_total, int block_tokens,
                       int max_pending, void* dev_pool, size_t pool_bytes, ee_kv_cache** out);
int ee_kv_cache_reset(ee_kv_cache* c, int seq); /* frees the sequence's blocks, clears its pending list */
/* Number of positions whose K,V are present in `layer` (0-based; n_layers + i: the layer inside exit i).  After an early exit the layers above the exit
 * lag behind the shallow ones (Section 4, "KV recomputation": the KV caches of the deep layers are missing for a
 * token that left early); the difference is what later steps, or a flush, fill in. */
int ee_kv_cache_filled(const ee_kv_cache* c, int seq, int layer, int32_t* n_positions);
/* Length of the sequence's list of deferred tokens (Section 4: the most recent tokens whose deep KV is missing). */
int ee_kv_cache_pending(const ee_kv_cache* c, int seq, int32_t* n_pending);
/* Copies K (after the rotary embedding) and V of positions [pos0, pos0+n) of one layer to host arrays
 * [n][d_model] fp32: the check that, after generation and a flush, the cache equals that of a full-depth pass over
 * the same tokens (Section 4: recomputation leaves no KV entry missing).  Blocks until the copy is done. */
int ee_kv_cache_read(ee_model* m, const ee_kv_cache* c, int seq, int layer, int pos0, int n, float* k_host,
                     float* v_host, void* stream);
/* Runs every deferred token of the given sequences through its missing layers; emits nothing (Section 4,
 * "KV recomputation": the deferred tokens go through a forward pass that fills their missing entries; here without
 * a current token, e.g. at the end of generation or before a step that would not fit).  Blocks until done. */
int ee_kv_cache_flush(ee_model* m, ee_kv_cache* c, int n_seqs, const int32_t* seq_ids, void* stream);
int ee_kv_cache_free(ee_kv_cache* c);

/* Pipeline-based early-exit inference on one GPU (Section 4, "Pipeline-based inference"; Appendix D.3; Appendix B.1:
 * both inference methods generate the same output).  With a second workspace and a second stream, the cache stops
 * deferring tokens: when a token leaves at an exit, ee_decode_step returns it at once and hands the token to
 * fill_stream, which carries it through the segments above the exit (the later pipeline stages) so that their KV
 * entries get filled, while the caller's stream already runs the next token's shallow segment.  A pass over a
 * segment on either stream waits (HIP events) for the latest pass over that segment on the other one, so a token
 * always finds the K and V of every earlier token.  The caller's lists stay empty: each sequence passes exactly
 * one row (its current token) per step, ee_kv_cache_pending reports 0 and no step is ever forced.
 *   dev_workspace   a second step workspace on the model's device, 256-byte aligned; workspace_bytes as reported by
 *                   ee_model_bytes is always enough (EE_ERR_NOMEM if too small).  NULL switches the mode off again.
 *   fill_stream     a HIP stream of the same priority as the one the steps are given, not the same stream.
 * Every token still passes every layer (on one stream or the other), so on one GPU this trades no work for the
 * early emission of tokens; ee_kv_cache_flush waits until the fill stream has caught up, and the read-backs and
 * ee_kv_cache_reset do so on their own.  At most four tokens are in flight on the fill stream; a step that would add
 * a fifth waits for the oldest.  EE_ERR_STATE while any token is deferred, EE_ERR_CONFIG in re-feed mode or when
 * the cache keeps fewer than 6 residual rows per sequence (max_pending < 5). */
int ee_kv_cache_set_pipeline(ee_model* m, ee_kv_cache* c, void* dev_workspace, size_t workspace_bytes, void* fill_stream);
/* Test hook: residual stream (fp32 [d_model]) of the sequence's newest processed position, at the
 * depth it reached. */
int ee_debug_read_hidden(ee_model* m, const ee_kv_cache* c, int seq, float* x_host, void* stream);

/* ---------------------------------------------------------------- prefill and decode */

/* Full-depth causal forward of a prompt into an empty sequence; all KV filled (the first token comes
 * from the prefill phase, Section 4).  The exit rule is then applied to the last position to choose
 * the first generated token: next_token / exit_layer follow the rule, conf[i] is the confidence at
 * exit i (i < n_exits) and conf[n_exits] at the final head; with threshold >= 1 the exits are not
 * evaluated and their conf entries are -1. */
int ee_prefill(ee_model* m, ee_kv_cache* c, int seq, const int32_t* tokens, int n_tokens, float threshold,
               int32_t* next_token, int32_t* exit_layer, float* conf, void* stream);

/* ee_prefill that also scores every head on EVERY prompt position (the per-token view of Table 4: which
 * token each exit would emit after each prefix, and how confident it is).  pos_token / pos_conf are host
 * arrays [n_exits+1][n_tokens] (row i < n_exits: exit i, last row: final head), filled whatever the
 * threshold: pos_token = arg max of the head's logits at that position (ties: lowest id), pos_conf = its
 * soft-max probability.  pos_nll (host, same shape, may be NULL): the negative log-likelihood each head gives
 * to the prompt's own next token, pos_nll[i][t] = log sum_v exp(z_v) - z[tokens[t+1]] for t < n_tokens-1 and 0 in
 * the last column: the per-token cross-entropy terms of the early-exit training objective (Section 3, Eq. (1):
 * a weighted sum of the exits' losses), computed from the same logits without storing them.
 * Everything else is as ee_prefill; row [.][n_tokens-1] repeats what the rule saw (to the precision of
 * ee_config::scored_head_terms: by default these heads read the leading bf16 term of their input only, which
 * moves a confidence by up to about 4e-3; the rule's own heads always read both).
 * Needs the prompt-phase GEMM path: a bf16 model with d_model a multiple of 128 (EE_ERR_CONFIG otherwise).
 * Prompts of 32 tokens or more, and every scored prompt, take that path: whole passes of up to
 * min(max_positions, prefill_rows) rows, rounded up to 128 (ee_config::prefill_rows), each projection one
 * matrix-core GEMM. */
int ee_prefill_scored(ee_model* m, ee_kv_cache* c, int seq, const int32_t* tokens, int n_tokens, float threshold,
                      int32_t* next_token, int32_t* exit_layer, float* conf, int32_t* pos_token, float* pos_conf,
                      float* pos_nll, void* stream);

/* One decode step for n_seqs sequences: early-exit inference with KV recomputation (Section 4, "KV
 * recomputation": the current token's pass also carries the recent tokens whose deep KV is missing; Section 5.2:
 * the confidence rule, tested at each exit in depth order; Appendix D.3: the list of deferred tokens and the forced
 * full pass once it has reached max_pending).  Blocks until the step's tokens are known.
 *   seq_ids      [n_seqs]   distinct sequence ids
 *   row_offsets  [n_seqs+1] rows of sequence i are tokens[row_offsets[i] .. row_offsets[i+1])
 *   tokens       per sequence: the ids of its deferred tokens, oldest first, then the current token
 *                (the one emitted by the previous call)
 *   pending_mask 1 = deferred row (KV fill only), 0 = current token; exactly the last row of each
 *                sequence is 0.  The library keeps the list itself and checks the caller's against
 *                it (EE_ERR_STATE on mismatch).
 *   threshold    exit iff confidence >= threshold and threshold < 1
 * Outputs, [n_seqs] each: next_token, exit_layer (an exit layer, or n_layers for a full or forced
 * step) and conf (confidence at the head that emitted).
 * With one sequence the call enqueues, behind each exit's head, the KV write and the attention of the next layer
 * before it knows the decision (they touch nothing a token that leaves depends on); when the token does leave, those
 * two kernels may still be running on `stream` as the call returns.  Later calls on the same stream are ordered behind
 * them; calls with this model on another stream wait for them first; ee_kv_cache_free and ee_model_free wait too.
 * Errors leave every sequence as it was: EE_ERR_STATE (rows disagree with the lists), EE_ERR_RANGE (token id,
 * position beyond max_positions), EE_ERR_NOMEM (no free cache block, or more rows than max_rows).  After an
 * EE_ERR_HIP (a launch failed, or the step's results did not arrive within two minutes) the handles must not be
 * used again. */
int ee_decode_step(ee_model* m, ee_kv_cache* c, int n_seqs, const int32_t* seq_ids, const int32_t* row_offsets,
                   const int32_t* tokens, const uint8_t* pending_mask, float threshold, int32_t* next_token,
                   int32_t* exit_layer, float* conf, void* stream);

/* ee_decode_step for callers that cannot provide (or allocate) a workspace at the time of the call: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same results bit for bit;
 * the step's workspace (descriptors, activations, attention and head partials) is not the buffer the model was
 * created over but an array of EE_STATIC_WORKSPACE_BYTES that the library keeps in each GPU's memory for the life of
 * the process.  The call allocates nothing, on the device or through any library.
 *   - EE_ERR_NOMEM, before anything is touched, if the model's decode workspace (the part of workspace_bytes in
 *     front of the prompt-phase buffers; it grows with max_rows, max_seqs, d_ff and vocab) is larger than that: the
 *     7B shape with max_rows <= 64 fits (28 MB), max_rows 256 (100 MB) does not.
 *   - EE_ERR_ARG if the current device is not the one that holds the model.
 *   - All calls on one GPU share the one array, whatever the model or the stream: two calls that overlap in time on
 *     the same GPU race.  The array keeps the last call's contents; a step reads nothing of it that the same step
 *     has not written first.
 * The prompt phase (ee_prefill) and ee_kv_cache_flush still use the model's own workspace. */
#define EE_STATIC_WORKSPACE_BYTES (32u << 20)
int ee_decode_step_static(ee_model* m, ee_kv_cache* c, int n_seqs, const int32_t* seq_ids, const int32_t* row_offsets,
                          const int32_t* tokens, const uint8_t* pending_mask, float threshold, int32_t* next_token,
                          int32_t* exit_layer, float* conf, void* stream);

#ifdef __cplusplus
}
#endif
#endif
