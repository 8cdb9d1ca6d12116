/*
 * CPU oracle for early-exit decoding with KV recomputation -- C API.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow reference that the HIP
 * library is checked against.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it; the product path never does.  It shares no
 * code, header, table or helper with the HIP library.
 *
 * What it computes (paper Section 4 "KV recomputation", Section 5.2 exit rule,
 * Appendix D.3 forced full pass, Appendix B.1 "both methods generate the same
 * output"):
 *   - G0: the plain definition.  Every new token is produced by a cache-free
 *     causal forward of the whole sequence so far; the exit rule is applied to
 *     the last position at each exit in depth order.
 *   - G1: the paper's mechanism.  A per-layer KV cache, a list of the most
 *     recent early-exited tokens whose deep KV is missing, and in every step
 *     those tokens are fed again with the current token (from layer 1) so that
 *     their KV is recomputed; a full-depth pass is forced when the list
 *     reaches max_pending.
 * Arithmetic: values are fp32; every reduction (dot product, mean square,
 * softmax sum) is one running fp64 sum in index order, rounded once to fp32;
 * a normalised vector is formed in fp64 (gain * x / root) and rounded once.  With
 * dtype = EO_BF16 the stored tensors are bf16: the weight matrices and the
 * embedding (given as bf16 bit patterns) and the cached K (after RoPE) and V,
 * which are rounded to bf16 (nearest even) when written.  Nothing else is
 * rounded: activations, the residual stream, q, softmax, logits and
 * confidences stay fp32.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * against closed forms, invariants, numpy/scipy fp64 routines and the G0
 * brute force (no "parity unpinned" function).
 */
#ifndef EE_ORACLE_H
#define EE_ORACLE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

enum { EO_F32 = 0, EO_BF16 = 1 };

typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ff, vocab;
    int32_t n_exits, exit_layers[8]; /* 1-based "after layer e", ascending, < n_layers */
    int32_t dtype;                   /* EO_F32 | EO_BF16: storage of matrices and the embedding */
    float rms_eps, rope_base;
    int32_t exit_flags;              /* EO_EXIT_* below; 0 = RMSNorm + own output embedding per exit */
} eo_config;

/* Structure of the exits (paper Section 2, "Model architectures": an output embedding matrix with an
 * optional normalisation in front of it, optionally preceded by an MLP; input and output embedding
 * matrices tied or untied):
 *   EO_EXIT_NO_NORM    exits apply their output embedding to the residual stream as it is (the final head
 *                      keeps its norm);
 *   EO_TIE_EMBEDDINGS  every exit and the final head use the input embedding matrix [vocab][d];
 *   EO_EXIT_MLP        exit i first applies an MLP block of its own, of the same form as a layer's:
 *                      x' = x + W_d (silu(W_g h) * (W_u h)), h = rmsnorm(x; g_mlp), and its (norm and)
 *                      output embedding read x'.  The backbone's x is not changed.
 *   EO_EXIT_LAYER      exit i first applies a complete Transformer layer of its own (the same block as a backbone
 *                      layer, own weights) to the hidden states at its depth: its attention at position t runs over
 *                      the K and V that this exit layer produced at positions 0..t.  Its output feeds the exit's
 *                      (norm and) output embedding; the backbone's x is not changed.  In generation with a KV cache,
 *                      every position that passes depth e_i leaves its K and V in the exit's layer (cache layer
 *                      n_layers + i), whether or not the exit is evaluated for it.  Not together with EO_EXIT_MLP. */
enum { EO_EXIT_NO_NORM = 1, EO_TIE_EMBEDDINGS = 2, EO_EXIT_MLP = 4, EO_EXIT_LAYER = 8 };

/* tensor kinds, same numbering as the workload generator's TensorKind */
enum { EO_EMBED = 0, EO_ATTN_NORM = 1, EO_WQ = 2, EO_WK = 3, EO_WV = 4, EO_WO = 5, EO_MLP_NORM = 6,
       EO_WG = 7, EO_WU = 8, EO_WD = 9, EO_EXIT_NORM = 10, EO_EXIT_HEAD = 11, EO_FINAL_NORM = 12,
       EO_FINAL_HEAD = 13, EO_EXIT_MLP_NORM = 14, EO_EXIT_WG = 15, EO_EXIT_WU = 16, EO_EXIT_WD = 17,
       /* attention half of an exit's Transformer layer; kinds 14..17 are its MLP half */
       EO_EXIT_ATTN_NORM = 18, EO_EXIT_WQ = 19, EO_EXIT_WK = 20, EO_EXIT_WV = 21, EO_EXIT_WO = 22 };

typedef struct eo_model eo_model;
typedef struct eo_state eo_state;

/* what one head evaluation saw (one row) */
typedef struct {
    int32_t layer;    /* depth of the head: exit layer e_i, or n_layers for the final head */
    int32_t argmax;   /* lowest index among maximal logits */
    int32_t arg2;     /* index of the runner-up logit */
    float conf;       /* max softmax probability = 1 / sum_i exp(z_i - z_max) */
    float top1, top2; /* the two largest logits */
} eo_diag;

void eo_set_threads(int n); /* row-parallel matvec threads (results do not depend on it); default 1 */
int eo_get_threads(void);

/* model: pointers are borrowed (the caller keeps the arrays alive).  Matrices/embedding: float* for
 * EO_F32, uint16_t* (bf16 bit patterns) for EO_BF16, row-major [out][in].  Norm gains: float*. */
eo_model* eo_model_create(const eo_config* cfg);
int eo_model_set_tensor(eo_model*, int kind, int index, const void* data);
void eo_model_free(eo_model*);

/* ---- G0: plain definition (cache-free) ---- */
/* Generates n_new tokens after the prompt; exit_layer_out[j] in {e_1.., n_layers}. */
int eo_generate_g0(const eo_model*, const int32_t* prompt, int n_prompt, int n_new, float threshold,
                   int32_t* tokens_out, int32_t* exit_layer_out);
/* Same, with the forced full-depth rule (Appendix D.3) derived from the exit history alone. */
int eo_generate_g0_capped(const eo_model*, const int32_t* prompt, int n_prompt, int n_new, float threshold,
                          int max_pending, int32_t* tokens_out, int32_t* exit_layer_out);
/* Exit-free greedy loop (a standard LLM): a third generator, used to pin threshold 1. */
int eo_generate_plain(const eo_model*, const int32_t* prompt, int n_prompt, int n_new, int32_t* tokens_out);
/* Cache-free forward of a whole sequence (layer-major).  Any output may be NULL.
 * hidden_out: [n_layers+1][n][d] residual stream after the embedding and after each layer.
 * k_out / v_out: [n_layers][n][d] keys (after RoPE) and values. */
int eo_forward_sequence(const eo_model*, const int32_t* tokens, int n, float* hidden_out, float* k_out,
                        float* v_out);

/* The Transformer layer of exit `exit` (EO_EXIT_LAYER) applied to a whole sequence of hidden states [n][d] (the
 * residual stream after layer e_i at positions 0..n-1), causally.  x_out: [n][d] its output; k_out / v_out: [n][d]
 * its keys (after RoPE) and values.  Any output may be NULL. */
int eo_exit_layer_sequence(const eo_model*, int exit, const float* hidden, int n, float* x_out, float* k_out, float* v_out);

/* ---- G1: KV cache + pending list + recomputation ---- */
eo_state* eo_state_create(const eo_model*, int max_positions, int max_pending);
void eo_state_free(eo_state*);
/* Full-depth forward of the prompt, all KV filled.  Every head is evaluated on the last position:
 * diag_out[0..n_exits-1] for the exits, diag_out[n_exits] for the final head. */
int eo_prefill(eo_state*, const int32_t* tokens, int n, eo_diag* diag_out);
/* One decode step in three parts, so that a test can drive the decision itself:
 *   begin   - takes the current token (the one emitted last); returns 1 if this step is forced full
 *             depth because the pending count has reached max_pending, else 0;
 *   advance - runs the next segment of layers over the pending rows and the current row; if the
 *             segment ends at an exit and eval_head != 0, or it ends at the last layer, evaluates
 *             that head on the current row into *diag.  Returns the depth reached;
 *   commit  - ends the step at the depth reached, emitting `token`. */
int eo_step_begin(eo_state*, int32_t token);
int eo_step_advance(eo_state*, int eval_head, eo_diag* diag);
int eo_step_commit(eo_state*, int32_t token);
/* The paper's rule on top of the three parts: exit at the first exit whose confidence >= threshold
 * (exits are not evaluated when threshold >= 1 or the step is forced). */
int eo_decode_step(eo_state*, int32_t token, float threshold, int32_t* next_token, int32_t* exit_layer,
                   float* conf);
/* Runs pending rows through their missing layers; no token is emitted. */
int eo_flush(eo_state*);
int eo_filled(const eo_state*, int segment); /* positions whose KV is present in every layer of the segment */
int eo_n_pending(const eo_state*);
int eo_kv_read(const eo_state*, int layer, int pos0, int n, float* k_out, float* v_out); /* [n][d]; layer n_layers + i: exit i's own layer */
int eo_last_hidden(const eo_state*, float* x_out); /* current row's residual stream at the depth reached */
int eo_last_logits(const eo_state*, float* z_out); /* logits of the last head evaluated, [vocab] */

/* ---- single operations, exported for pins and real-shape spot checks ---- */
float eo_bf16_round(float v);
/* y = W rmsnorm(x; g), rmsnorm(x; g)[k] = g[k] x[k] / sqrt(mean(x^2)+eps); g == NULL: no norm, y = W x */
void eo_norm_matvec(int dtype, const void* W, int N, int K, const float* x, const float* g, float eps,
                    float* y);
void eo_rope(float* vec, int n_heads, int head_dim, int pos, float base);
/* one query row over n_ctx cached positions; q,out: [H*hd]; K,V: [n_ctx][H*hd] */
void eo_attention_row(const float* q, const float* K, const float* V, int n_ctx, int n_heads,
                      int head_dim, float* out);
void eo_swiglu(const float* gate, const float* up, int n, float* out);
void eo_softmax_max(const float* z, int n, eo_diag* out);
/* one layer on one row: x in/out [d]; K,V: [>=pos+1][d], row `pos` is written, rows 0..pos are read */
int eo_layer_row(const eo_model*, int layer, float* x, int pos, float* K, float* V);
/* head i (0..n_exits-1 exits, n_exits = final) on one row; z_out may be NULL.  For a model with EO_EXIT_LAYER, x is
 * the output of the exit's layer at that row (eo_exit_layer_sequence): this call applies what comes after it. */
int eo_head_row(const eo_model*, int head, const float* x, float* z_out, eo_diag* diag);

#ifdef __cplusplus
}
#endif
#endif
