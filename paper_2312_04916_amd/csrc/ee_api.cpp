// Host side of the C ABI declared in ee.h: buffer layout, weight packing, the paged KV cache with its
// per-sequence fill watermarks and list of deferred tokens, and the step scheduler that launches one
// segment of layers at a time and reads the exit decision back before launching the next
// (Section 4 "KV recomputation", Section 5.2 exit rule, Appendix D.3 forced full pass).
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "ee_internal.h"
#include "ee_plan.h"

using namespace ee;

namespace {

thread_local int g_last_hip = 0;

#define HIPCHK(expr)                          \
    do {                                      \
        hipError_t _e = (expr);               \
        if (_e != hipSuccess) {               \
            g_last_hip = (int)_e;             \
            return EE_ERR_HIP;                \
        }                                     \
    } while (0)

#define EECHK(expr)              \
    do {                         \
        int _r = (expr);         \
        if (_r != EE_OK) return _r; \
    } while (0)

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline size_t esize(int dtype) { return dtype == EE_BF16 ? 2 : 4; }

int check_config(const ee_config& c) {
    if (c.n_layers < 1 || c.n_heads < 1 || c.d_model != c.n_heads * c.head_dim) return EE_ERR_CONFIG;
    if (c.head_dim != 32 && c.head_dim != 64 && c.head_dim != 128) return EE_ERR_CONFIG;
    if (c.d_model % 32 || c.d_ff % 32 || c.d_ff < 32 || c.vocab % 32 || c.vocab < 32) return EE_ERR_CONFIG;
    if (c.dtype != EE_F32 && c.dtype != EE_BF16) return EE_ERR_CONFIG;
    if (c.n_exits < 0 || c.n_exits > EE_MAX_EXITS) return EE_ERR_CONFIG;
    for (int i = 0; i < c.n_exits; ++i) {
        if (c.exit_layers[i] < 1 || c.exit_layers[i] >= c.n_layers) return EE_ERR_CONFIG;
        if (i && c.exit_layers[i] <= c.exit_layers[i - 1]) return EE_ERR_CONFIG;
    }
    if (c.max_positions < 1 || c.max_positions > (1 << 20)) return EE_ERR_CONFIG;
    if (!(c.rms_eps > 0.f) || !(c.rope_base > 1.f)) return EE_ERR_CONFIG;
    if (c.exit_flags & ~(EE_EXIT_NO_NORM | EE_TIE_EMBEDDINGS | EE_EXIT_MLP | EE_EXIT_LAYER)) return EE_ERR_CONFIG;
    if ((c.exit_flags & EE_EXIT_MLP) && (c.exit_flags & EE_EXIT_LAYER)) return EE_ERR_CONFIG;
    if (c.gemm_min_workgroups < 0 || c.scored_head_terms < 0 || c.scored_head_terms > 2) return EE_ERR_CONFIG;
    return EE_OK;
}

struct WeightLayout {
    size_t embed, rope, gf, wf, ones, total;
    std::vector<size_t> g1, qkv, wo, g2, gu, wd, ge, we;
    std::vector<size_t> gm, egu, ewd;  // exits with an MLP (or a whole layer): its norm gain, gate|up, down
    std::vector<size_t> ga, eqkv, ewo; // exits with a whole layer: attention norm gain, q|k|v, o
};

WeightLayout weight_layout(const ee_config& c) {
    WeightLayout w;
    size_t es = esize(c.dtype), d = c.d_model, F = c.d_ff, V = c.vocab, off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += align_up(bytes);
        return o;
    };
    w.embed = take(V * d * es);
    for (int l = 0; l < c.n_layers; ++l) {
        w.g1.push_back(take(d * 4));
        w.qkv.push_back(take(3 * d * d * es));
        w.wo.push_back(take(d * d * es));
        w.g2.push_back(take(d * 4));
        w.gu.push_back(take(2 * F * d * es));
        w.wd.push_back(take(d * F * es));
    }
    const bool tied = c.exit_flags & EE_TIE_EMBEDDINGS;
    for (int i = 0; i < c.n_exits; ++i) {
        if (c.exit_flags & EE_EXIT_LAYER) {
            w.ga.push_back(take(d * 4));
            w.eqkv.push_back(take(3 * d * d * es));
            w.ewo.push_back(take(d * d * es));
        }
        if (c.exit_flags & (EE_EXIT_MLP | EE_EXIT_LAYER)) {
            w.gm.push_back(take(d * 4));
            w.egu.push_back(take(2 * F * d * es));
            w.ewd.push_back(take(d * F * es));
        }
        w.ge.push_back(take(d * 4));
        if (!tied) w.we.push_back(take(V * d * es));
    }
    w.gf = take(d * 4);
    w.wf = take(V * d * es);  // tied embeddings: the one matrix every head reads, in the GEMM's tile order
    if (tied) w.we.assign(c.n_exits, w.wf);
    w.ones = take(d * 4);     // a gain of 1 for exits without a norm
    w.rope = take((size_t)c.max_positions * (c.head_dim / 2) * 8);
    w.total = off;
    return w;
}

struct WorkspaceLayout {
    size_t upload, upload_bytes;  // [descs][btab][tokens], one host-to-device copy per step
    size_t descs, btab, tokens;
    size_t q, attn, act, xg_pk, head_pk, partials, counters, attn_part, stage, total;
    int max_blocks_per_seq;
    // prompt phase (bf16 model): buffers for pf_rows positions at a time, activations in the packed operand layout
    int pf_rows;  // 0: the prompt phase runs through the decode kernels in chunks
    size_t pf_begin, pf_tokens, pf_x, pf_xg, pf_xgh, pf_q, pf_attn, pf_act, pf_ssq, pf_ssqe, pf_partials, pf_tok, pf_conf, pf_tgt, pf_zt, pf_nll;
};

// Rows per pass of the prompt-phase GEMM path; 0 when the model does not qualify (fp32, or widths the
// 256-column tiles do not divide evenly into the q|k|v parts).  ee_config::prefill_rows caps it (default 2048).
constexpr int PF_MIN_TOKENS = 32;  // shorter prompts go through the decode kernels

int pf_rows_of(const ee_config& c) {
    if (c.dtype != EE_BF16 || c.d_model % 128 || c.prefill_rows < 0) return 0;
    const int cap = c.prefill_rows == 0 ? 2048 : std::max(128, std::min(c.prefill_rows, 8192));
    int r = std::min((c.max_positions + 127) / 128 * 128, cap);
    return r / 128 * 128;
}

inline size_t rows_padded(int max_rows) { return ((size_t)max_rows + 63) / 64 * 64; }

WorkspaceLayout workspace_layout(const ee_config& c, int max_rows, int max_seqs) {
    WorkspaceLayout w;
    size_t es = esize(c.dtype), d = c.d_model, off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += align_up(bytes);
        return o;
    };
    w.max_blocks_per_seq = c.max_positions / 32 + 1;
    w.upload = off;
    // one descriptor per segment; with an MLP or a layer in the exits, one more per segment for the rows that works on
    w.descs = take(sizeof(SegDesc) * (EE_MAX_EXITS + 1) * ((c.exit_flags & (EE_EXIT_MLP | EE_EXIT_LAYER)) ? 2 : 1));
    w.btab = take((size_t)max_seqs * w.max_blocks_per_seq * 4);
    w.tokens = take(EE_MAX_ROWS * 4);
    w.upload_bytes = off - w.upload;
    size_t terms = c.dtype == EE_BF16 ? 2 : 1;  // bf16 activations are stored as hi and lo terms
    size_t rows = rows_padded(max_rows);        // (packed arrays hold whole groups of 16 rows)
    w.q = take(terms * rows * d * es);
    w.attn = take(terms * rows * d * es);
    w.act = take(terms * rows * c.d_ff * es);
    w.xg_pk = take(terms * rows * d * es);
    w.head_pk = take(terms * 64 * d * es);
    w.partials = take((size_t)(c.vocab / 16) * EE_MAX_SEQS * sizeof(HeadPartial));
    w.counters = take(256 * 4);
    w.attn_part = take(attention_part_floats(max_rows, c.n_heads, c.head_dim) * 4);
    w.stage = take(2 * (size_t)max_rows * d * 4);
    w.pf_rows = pf_rows_of(c);
    w.pf_begin = off;
    if (w.pf_rows) {
        size_t Mp = w.pf_rows, F = c.d_ff;
        w.pf_tokens = take(Mp * 4);
        w.pf_x = take(Mp * d * 4);
        w.pf_xg = take(2 * Mp * d * 2);
        w.pf_xgh = take(2 * Mp * d * 2);
        w.pf_q = take(2 * Mp * d * 2);
        w.pf_attn = take(2 * Mp * d * 2);
        w.pf_act = take(2 * Mp * F * 2);
        w.pf_ssq = take(Mp * ((d + 255) / 256) * 4);
        w.pf_ssqe = take(Mp * ((d + 255) / 256) * 4);  // the same for the rows an exit's MLP has changed
        w.pf_partials = take(Mp * (((size_t)c.vocab + 255) / 256) * sizeof(HeadPartial));
        w.pf_tok = take(Mp * 4);
        w.pf_conf = take(Mp * 4);
        w.pf_tgt = take(Mp * 4);   // per row: the next token of the prompt (scoring its log-likelihood)
        w.pf_zt = take(Mp * 4);    // its logit
        w.pf_nll = take(Mp * 4);
    }
    w.total = off;
    return w;
}

}  // namespace

struct ee_model {
    ee_config cfg;
    int max_rows, max_seqs;
    char* wbase;
    char* ws;
    WeightLayout wl;
    WorkspaceLayout wsl;
    std::vector<uint8_t> have;  // per tensor: set?
    int n_missing;
    char* pinned;            // host staging for the upload region, then the head results
    char* pinned_dev;        // device view of the same memory
    HeadResult* results;     // host view
    HeadResult* results_dev; // device view of the same memory
    int32_t* pf_host_tokens; // pinned staging of one prompt pass's token ids
    int head_tag = 0;        // tag of the latest head evaluation (see HeadResult::pad)
    int head_wait_limit_s = 120;  // wall-clock bound of one wait for head results
    int step_tag0 = 0;            // head_tag when the latest decode step began: later tags belong to that step
    float* dbg_logits;
    int dbg_rows;
    int prof_kernel = -1;               // kernel family being timed, or -1
    int prof_every = 1, prof_seen = 0;  // every prof_every-th launch of the family is timed
    // A decode step at batch 1 enqueues the first two kernels of the next segment before it knows whether the token
    // leaves at the exit (run_step); when it does leave, they are still running on `spec_stream` as the call returns.
    // Work on the same stream is ordered behind them anyway; a call on another stream waits for `spec_ev` first.
    hipEvent_t spec_ev = nullptr;
    hipStream_t spec_stream = nullptr;
    bool spec_recorded = false;
    std::vector<hipEvent_t> prof_ev;    // event pairs
    size_t prof_used = 0;               // events recorded so far
    size_t lo_rows(size_t ld) const { return cfg.dtype == EE_BF16 ? rows_padded(max_rows) * ld : 0; }  // hi -> lo distance
    int n_seg() const { return cfg.n_exits + 1; }
    int seg_begin(int s) const { return s == 0 ? 0 : cfg.exit_layers[s - 1]; }
    int seg_end(int s) const { return s < cfg.n_exits ? cfg.exit_layers[s] : cfg.n_layers; }
    int seg_of_layer(int l) const {
        for (int s = 0; s < n_seg(); ++s)
            if (l < seg_end(s)) return s;
        return n_seg() - 1;
    }
    SegDesc* host_desc(int i) const { return (SegDesc*)(pinned + (wsl.descs - wsl.upload)) + i; }
    int32_t* host_btab() const { return (int32_t*)(pinned + (wsl.btab - wsl.upload)); }
    int32_t* host_tokens() const { return (int32_t*)(pinned + (wsl.tokens - wsl.upload)); }
    SegDesc* dev_desc(int i) const { return (SegDesc*)(ws + wsl.descs) + i; }
    int32_t* dev_btab() const { return (int32_t*)(ws + wsl.btab); }
    int32_t* dev_tokens() const { return (int32_t*)(ws + wsl.tokens); }
    const float* gain(size_t off) const { return (const float*)(wbase + off); }
    int tensor_slot(int kind, int index) const {
        int L = cfg.n_layers, E = cfg.n_exits;
        switch (kind) {
            case EE_T_EMBED: return index == 0 ? 0 : -1;
            case EE_T_FINAL_NORM: return index == 0 ? 1 : -1;
            case EE_T_FINAL_HEAD: return index == 0 ? 2 : -1;
            case EE_T_EXIT_NORM: return index >= 0 && index < E ? 3 + index : -1;
            case EE_T_EXIT_HEAD: return index >= 0 && index < E ? 3 + E + index : -1;
            default: break;
        }
        static const int per_layer[] = {EE_T_ATTN_NORM, EE_T_WQ, EE_T_WK, EE_T_WV, EE_T_WO, EE_T_MLP_NORM, EE_T_WG, EE_T_WU, EE_T_WD};
        for (int j = 0; j < 9; ++j)
            if (per_layer[j] == kind) return index >= 0 && index < L ? 3 + 2 * E + index * 9 + j : -1;
        static const int per_exit[] = {EE_T_EXIT_MLP_NORM, EE_T_EXIT_WG, EE_T_EXIT_WU, EE_T_EXIT_WD, EE_T_EXIT_ATTN_NORM,
                                       EE_T_EXIT_WQ,       EE_T_EXIT_WK, EE_T_EXIT_WV,       EE_T_EXIT_WO};
        for (int j = 0; j < 9; ++j)
            if (per_exit[j] == kind) return index >= 0 && index < E ? 3 + 2 * E + 9 * L + index * 9 + j : -1;
        return -1;
    }
    int n_tensors() const { return 3 + 2 * cfg.n_exits + 9 * cfg.n_layers + 9 * cfg.n_exits; }
    bool exit_mlp() const { return cfg.exit_flags & EE_EXIT_MLP; }
    bool exit_layer() const { return cfg.exit_flags & EE_EXIT_LAYER; }
    bool exit_block() const { return exit_mlp() || exit_layer(); }  // the exit works on copies of its rows
    int n_kv_layers() const { return cfg.n_layers + (exit_layer() ? cfg.n_exits : 0); }  // exit i's layer caches as layer L+i
    int mlp_desc(int seg) const { return EE_MAX_EXITS + 1 + seg; }  // descriptor of the rows exit `seg`'s MLP works on
    bool exit_norm() const { return !(cfg.exit_flags & EE_EXIT_NO_NORM); }
    bool tied() const { return cfg.exit_flags & EE_TIE_EMBEDDINGS; }
    // is this tensor part of the model as configured?
    bool applicable(int kind) const {
        switch (kind) {
            case EE_T_EXIT_NORM: return exit_norm();
            case EE_T_EXIT_HEAD:
            case EE_T_FINAL_HEAD: return !tied();
            case EE_T_EXIT_MLP_NORM:
            case EE_T_EXIT_WG:
            case EE_T_EXIT_WU:
            case EE_T_EXIT_WD: return exit_block();
            case EE_T_EXIT_ATTN_NORM:
            case EE_T_EXIT_WQ:
            case EE_T_EXIT_WK:
            case EE_T_EXIT_WV:
            case EE_T_EXIT_WO: return exit_layer();
            default: return true;
        }
    }
    // gain folded into the operand that exit i reads first (its layer's or MLP's first norm, else its own norm, else none)
    const float* exit_in_gain(int i) const {
        return gain(exit_layer() ? wl.ga[i] : exit_mlp() ? wl.gm[i] : (exit_norm() ? wl.ge[i] : wl.ones));
    }
    // gain in front of exit i's output embedding
    const float* exit_out_gain(int i) const { return gain(exit_norm() ? wl.ge[i] : wl.ones); }
};

struct SeqState {
    std::vector<int32_t> filled;   // per segment: positions whose KV is present in all its layers
    std::vector<int32_t> blocks;   // logical block -> physical block
    std::vector<int32_t> tokring;  // token id of position p at p % S
};

// Pipeline-based early exit on one GPU (Section 4, "Pipeline-based inference"; Appendix D.3): a token that leaves at an
// exit is handed to a second stream, which runs it through its remaining segments (stages) to fill their KV
// entries while the caller's stream already works on the next token.  A pass over segment k on one stream waits for
// the latest pass over segment k on the other (the stage's earlier token), so every token finds the KV of its
// predecessors.  The second stream has its own step workspace and a ring of host staging areas for its descriptors.
struct Pipeline {
    static constexpr int RING = 4, POOL = 256;
    bool on = false;
    hipStream_t stream = nullptr;   // the fill stream
    char* ws = nullptr;             // its step workspace (device)
    char* pinned = nullptr;         // RING staging areas (host, mapped)
    char* pinned_dev = nullptr;
    size_t slot_bytes = 0;
    int next_slot = 0;
    bool slot_used[RING] = {};
    hipEvent_t slot_done[RING] = {};  // the fill that read staging area i has run
    hipEvent_t pool[POOL] = {};       // pass-finished events, handed out round-robin
    int next_ev = 0;
    int last_ev[EE_MAX_EXITS + 1];    // per segment: pool index of its latest pass, or -1
    hipStream_t last_stream[EE_MAX_EXITS + 1];
    bool events_made = false;
};

struct ee_kv_cache {
    const ee_model* m;
    int max_seqs, BT, S, max_pending, n_blocks;
    int refeed = 0;  // deferred tokens re-enter at layer 1 (the paper's wording) instead of resuming where they stopped
    bool spec_used = false;  // a decode step on this cache has left kernels in flight at its return (see run_step)
    Pipeline pipe;
    char* pool;
    size_t off_x, off_xg, off_xgh, off_ssq;
    size_t xs_lo;    // element distance from the hi to the lo term in xg / xgh (0 for fp32)
    int ssq_stride;  // partial sums per row
    KvGeom geom;
    std::vector<int32_t> free_blocks;
    std::vector<SeqState> seqs;
    float* x() const { return (float*)(pool + off_x); }
    void* xg() const { return pool + off_xg; }
    void* xgh() const { return pool + off_xgh; }
    float* ssq() const { return (float*)(pool + off_ssq); }
    int slot_of(int seq, int pos) const { return seq * S + pos % S; }
    int transient_slot(int r) const { return max_seqs * S + r; }
    int exit_slot(int r) const { return max_seqs * S + m->max_rows + r; }  // copies an exit's MLP or layer works on
    int n_pending(const SeqState& s) const { return plan::pending(s.filled.data(), (int)s.filled.size()); }
};

namespace {

// rows of the residual store: one per position a sequence may have deferred plus its current one, the transient rows
// of a prompt chunk, and the copies that exits with an MLP work on
// Residual rows kept per sequence: its deferred tokens and the current one.  Without a cap (max_pending <= 0) the
// list is bounded by what one step can carry: max_rows rows.
int slots_per_seq(const ee_model* m, int max_pending) { return max_pending > 0 ? max_pending + 1 : m->max_rows; }

size_t store_slots(const ee_model* m, int max_seqs, int max_pending) {
    // (an exit's MLP works on copies of the head rows, an exit's layer on copies of all the rows of the launch)
    return (size_t)max_seqs * slots_per_seq(m, max_pending) + m->max_rows + (m->exit_layer() ? m->max_rows : m->exit_mlp() ? m->max_seqs : 0);
}

size_t kv_pool_layout(const ee_model* m, int max_seqs, int64_t max_tokens_total, int BT, int max_pending, int* n_blocks,
                      size_t* off_x, size_t* off_xg, size_t* off_xgh, size_t* off_ssq) {
    const ee_config& c = m->cfg;
    size_t es = esize(c.dtype), d = c.d_model;
    int nb = (int)((max_tokens_total + BT - 1) / BT) + max_seqs;
    size_t blk = 2 * (size_t)c.n_heads * BT * c.head_dim;
    size_t off = align_up((size_t)m->n_kv_layers() * nb * blk * es);
    size_t slots = store_slots(m, max_seqs, max_pending);
    size_t P = d / (16 * gemm_resid_tiles_per_wg());
    if (n_blocks) *n_blocks = nb;
    if (off_x) *off_x = off;
    off += align_up(slots * d * 4);
    size_t terms = c.dtype == EE_BF16 ? 2 : 1;
    if (off_xg) *off_xg = off;
    off += align_up(terms * slots * d * es);
    if (off_xgh) *off_xgh = off;
    off += align_up(terms * slots * d * es);
    if (off_ssq) *off_ssq = off;
    off += align_up(slots * P * 4);
    return off;
}

int check_cache_args(const ee_model* m, int max_seqs, int64_t max_tokens_total, int BT, int max_pending) {
    if (!m) return EE_ERR_ARG;
    if (max_seqs < 1 || max_seqs > 4096 || max_tokens_total < 1 || BT < 32 || BT % 32 || BT > 1024) return EE_ERR_CONFIG;
    if (max_pending > EE_MAX_ROWS - 1) return EE_ERR_CONFIG;
    return EE_OK;
}

// Attaches an event pair to the next launch when its kernel family is being timed.
struct Timed {
    Timed(ee_model* m, int kernel, hipStream_t) {
        if (m->prof_kernel == kernel && m->prof_seen++ % m->prof_every == 0 && m->prof_used + 2 <= m->prof_ev.size()) {
            set_launch_events(m->prof_ev[m->prof_used], m->prof_ev[m->prof_used + 1]);
            m->prof_used += 2;
        }
    }
};

// The MLP half of a block over the rows of g.desc: x += W_d (silu(W_g h) * (W_u h)), h = the rows' x.g operand in
// `a_src` (slots `arow`) scaled by their RMS.  Leaves x.g_next (and x.g_head in the second operand store when
// g_head is given) and the sum-of-squares partials of the new x.  Used by every layer and by exits with an MLP.
int run_mlp(ee_model* m, ee_kv_cache* c, GemmCommon g, const char* w_gu, const char* w_d, void* a_src, const int32_t* arow, bool pk_d,
            bool pk_F, const float* g_next, const float* g_head, bool pack_next, hipStream_t st) {
    const ee_config& cf = m->cfg;
    const int d = cf.d_model, F = cf.d_ff;
    char* xg_pk = m->ws + m->wsl.xg_pk;
    // act = silu(W_g h) * (W_u h)
    g.W = w_gu;
    g.N = 2 * F;
    g.K = d;
    g.A = pk_d ? (void*)xg_pk : a_src;
    g.a_lo = pk_d ? m->lo_rows(d) : c->xs_lo;
    g.a_packed = pk_d;
    g.lda = d;
    g.arow = arow;
    g.ssq = c->ssq();
    {
        Timed t(m, EE_K_SWIGLU, st);
        HIPCHK(launch_gemm_swiglu(g, m->ws + m->wsl.act, m->lo_rows(F), F, pk_F, st));
    }
    // x += W_d act ; operand for what reads x next
    g.W = w_d;
    g.N = d;
    g.K = F;
    g.A = m->ws + m->wsl.act;
    g.a_lo = m->lo_rows(F);
    g.a_packed = pk_F;
    g.lda = F;
    g.arow = nullptr;
    g.ssq = nullptr;
    {
        Timed t(m, EE_K_DOWN, st);
        HIPCHK(launch_gemm_resid(g, c->x(), c->xg(), g_head ? c->xgh() : nullptr, c->xs_lo, c->ssq(), g_next, g_head, d,
                                 pack_next ? xg_pk : nullptr, m->lo_rows(d), st));
    }
    return EE_OK;
}

// The weights of one Transformer block: a backbone layer, or the layer an exit may contain.
struct BlockW {
    const char *qkv, *wo, *gu, *wd;
    const float* g2;  // gain of the norm in front of the MLP half
};

// One block over the rows described by dev_desc(di): q,k,v = W_qkv rmsnorm(x; g1) with rotary embedding and the KV
// write into cache layer kv_layer, attention, x += W_o a, the MLP half.  The rows' x.g1 operand is read from `a_first`
// (a row-major operand store, indexed by the rows' slots), or from the packed copy when the rows are too many for LDS
// (the caller has packed it).  kv_only: stop after the KV write (the rows only have to leave their K and V here).
enum { BLOCK_ALL = 0, BLOCK_FRONT = 1, BLOCK_REST = 2 };  // FRONT: the KV write and the attention; REST: what follows them

int run_block(ee_model* m, ee_kv_cache* c, int di, int T, int n_qt, int kv_layer, const BlockW& w, void* a_first, bool kv_only,
              const float* g_next, const float* g_head, bool pack_next, int max_ctx, hipStream_t st, int phase = BLOCK_ALL,
              int* att_ns_io = nullptr) {
    const ee_config& cf = m->cfg;
    const int d = cf.d_model, F = cf.d_ff, dt = cf.dtype;
    SegDesc* dd = m->dev_desc(di);
    const int32_t* xrow = (const int32_t*)((char*)dd + offsetof(SegDesc, xrow));
    const bool pk_d = dt == EE_BF16 && !gemm_rows_fit_lds(dt, T, d);
    const bool pk_F = dt == EE_BF16 && !gemm_rows_fit_lds(dt, T, F);
    char* xg_pk = m->ws + m->wsl.xg_pk;
    GemmCommon g{};
    g.dtype = dt;
    g.T = T;
    g.min_wgs = cf.gemm_min_workgroups;
    g.desc = dd;
    g.desc_host = m->host_desc(di);
    g.inv_d = 1.0f / (float)d;
    g.eps = cf.rms_eps;
    g.ssq_stride = c->ssq_stride;
    g.ssq_n = c->ssq_stride;
    // q,k,v = W_qkv rmsnorm(x; g1); rotary; KV write
    g.W = w.qkv;
    g.N = 3 * d;
    g.K = d;
    g.A = pk_d ? (void*)xg_pk : a_first;
    g.a_lo = pk_d ? m->lo_rows(d) : c->xs_lo;
    g.a_packed = pk_d;
    g.lda = d;
    g.arow = xrow;
    g.ssq = c->ssq();
    if (phase != BLOCK_REST) {
        Timed t(m, EE_K_QKV, st);
        HIPCHK(launch_gemm_qkv(g, m->ws + m->wsl.q, m->lo_rows(d), (const float*)(m->wbase + m->wl.rope), c->geom, kv_layer, st));
    }
    if (kv_only) return EE_OK;
    int att_ns = phase == BLOCK_REST ? *att_ns_io : 0;
    if (phase != BLOCK_REST) {
        Timed t(m, EE_K_ATTN, st);
        HIPCHK(launch_attention(dt, m->ws + m->wsl.q, m->ws + m->wsl.attn, m->lo_rows(d), dd, g.desc_host, T, n_qt, m->dev_btab(), c->geom,
                                kv_layer, d,
                                (float*)(m->ws + m->wsl.attn_part), (int32_t*)(m->ws + m->wsl.counters) + 64, max_ctx,
                                gemm_rows_fit_lds(dt, T, d) ? &att_ns : nullptr, pk_d, st));
    }
    if (phase == BLOCK_FRONT) {
        *att_ns_io = att_ns;
        return EE_OK;
    }
    // x += W_o a ; operand for the MLP norm
    g.W = w.wo;
    g.N = d;
    g.K = d;
    g.A = m->ws + m->wsl.attn;
    g.a_lo = m->lo_rows(d);
    g.a_packed = pk_d;
    g.arow = nullptr;
    g.ssq = nullptr;
    if (att_ns > 0) {
        g.att_part = (const float*)(m->ws + m->wsl.attn_part);
        g.att_ns = att_ns;
        g.att_H = cf.n_heads;
        g.att_hd = cf.head_dim;
    }
    {
        Timed t(m, EE_K_OPROJ, st);
        HIPCHK(launch_gemm_resid(g, c->x(), c->xg(), nullptr, c->xs_lo, c->ssq(), w.g2, nullptr, d, pk_d ? xg_pk : nullptr,
                                 m->lo_rows(d), st));
    }
    g.att_part = nullptr;
    // (the next block of this call reads the packed copy; across calls the residual store is the interface)
    return run_mlp(m, c, g, w.gu, w.wd, c->xg(), xrow, pk_d, pk_F, g_next, g_head, pk_d && pack_next, st);
}

// ---- the per-layer launch sequence over the rows described by dev_desc(di)
// first_phase: BLOCK_FRONT stops after the attention of layer l0 (nothing of the rows' residual stream has changed
// then); BLOCK_REST takes the pass up from there.  *att_ns_io carries the attention's split count between the two.
int run_layers(ee_model* m, ee_kv_cache* c, int di, int T, int n_qt, int l0, int l1, int max_ctx, hipStream_t st,
               int first_phase = BLOCK_ALL, int* att_ns_io = nullptr) {
    const ee_config& cf = m->cfg;
    const int d = cf.d_model, dt = cf.dtype;
    SegDesc* dd = m->dev_desc(di);
    const int32_t* xrow = (const int32_t*)((char*)dd + offsetof(SegDesc, xrow));
    // More rows than a workgroup can stage in LDS: the GEMMs then take their row operands from packed arrays
    // (dense rows of this launch in MFMA operand order) that the producing epilogues write, and the segment
    // starts by packing the rows' x.g operands out of the residual store.
    const bool pk_d = dt == EE_BF16 && !gemm_rows_fit_lds(dt, T, d);
    if (pk_d && l0 < l1 && first_phase != BLOCK_REST)
        HIPCHK(launch_pack_rows(c->xg(), c->xs_lo, d, xrow, T, d, m->ws + m->wsl.xg_pk, m->lo_rows(d), st));
    for (int l = l0; l < l1; ++l) {
        const BlockW w{m->wbase + m->wl.qkv[l], m->wbase + m->wl.wo[l], m->wbase + m->wl.gu[l], m->wbase + m->wl.wd[l],
                       m->gain(m->wl.g2[l])};
        const float* g_next = (l + 1 < cf.n_layers) ? m->gain(m->wl.g1[l + 1]) : m->gain(m->wl.gf);
        const float* g_head = nullptr;
        for (int i = 0; i < cf.n_exits; ++i)
            if (cf.exit_layers[i] == l + 1) g_head = m->exit_in_gain(i);
        EECHK(run_block(m, c, di, T, n_qt, l, w, c->xg(), false, g_next, g_head, l + 1 < l1, max_ctx, st,
                        l == l0 ? first_phase : BLOCK_ALL, att_ns_io));
        if (l == l0 && first_phase == BLOCK_FRONT) break;
    }
    return EE_OK;
}

// Rows that exit `seg`'s MLP works on: copies, in slots of their own, of the head rows listed in host_desc(seg).
// Call after the head rows of host_desc(seg) are set and before the descriptors are uploaded.
void fill_exit_layer_desc(const ee_model* m, const ee_kv_cache* c, int seg, const SegDesc* d);

void fill_mlp_desc(const ee_model* m, const ee_kv_cache* c, int seg) {
    if (seg >= m->cfg.n_exits) return;
    if (m->exit_layer()) fill_exit_layer_desc(m, c, seg, m->host_desc(seg));
    if (!m->exit_mlp()) return;
    const SegDesc* d = m->host_desc(seg);
    SegDesc* e = m->host_desc(m->mlp_desc(seg));
    e->T = d->n_head;
    e->n_qt = 0;
    e->n_head = d->n_head;
    e->pad = 0;
    for (int r = 0; r < d->n_head; ++r) {
        e->xrow[r] = c->exit_slot(r);
        e->row_qt[r] = r;
        e->pos[r] = e->kvblk[r] = e->rseq[r] = 0;
        e->head_xrow[r] = c->exit_slot(r);
        e->head_slot[r] = d->head_slot[r];
    }
}

// Rows that exit `seg`'s own Transformer layer works on: copies, in slots of their own, of ALL the rows of `d` (each
// leaves its K and V in the exit's layer), at the same positions; the head rows are the copies of d's head rows.
void fill_exit_layer_desc(const ee_model* m, const ee_kv_cache* c, int seg, const SegDesc* d) {
    SegDesc* e = m->host_desc(m->mlp_desc(seg));
    if (e != d) *e = *d;  // positions, cache blocks, sequences and query tiles are those of the rows copied
    for (int r = 0; r < d->T; ++r) e->xrow[r] = c->exit_slot(r);
    for (int j = 0; j < d->n_head; ++j) {
        int r = 0;
        while (r < d->T && d->xrow[r] != d->head_xrow[j]) ++r;
        e->head_xrow[j] = c->exit_slot(r < d->T ? r : 0);
    }
}

// The Transformer layer inside exit `seg` over the rows whose residual-store slots are listed in the device array
// `src` (host_desc(mlp_desc(seg)) lists their copies): the rows' x, first operand and sum-of-squares partials are copied to the exit's slots, every copy leaves
// its K and V in the exit's cache layer, and, with_head, the whole layer runs on the copies so that the head rows'
// x'.g (g: the exit's norm gain, or 1) stands in the first operand store at the copies' slots.
int run_exit_layer(ee_model* m, ee_kv_cache* c, int seg, const int32_t* src, bool with_head, int max_ctx, hipStream_t st) {
    const ee_config& cf = m->cfg;
    const int d = cf.d_model, dt = cf.dtype, me = m->mlp_desc(seg);
    const SegDesc* eh = m->host_desc(me);
    const int T = eh->T;
    if (T <= 0) return EE_OK;
    const int32_t* dst = (const int32_t*)((char*)m->dev_desc(me) + offsetof(SegDesc, xrow));
    HIPCHK(launch_copy_slots(dt, src, dst, T, d, c->x(), c->xgh(), c->xs_lo, c->ssq(), c->ssq_stride, st));
    if (dt == EE_BF16 && !gemm_rows_fit_lds(dt, T, d))
        HIPCHK(launch_pack_rows(c->xgh(), c->xs_lo, d, dst, T, d, m->ws + m->wsl.xg_pk, m->lo_rows(d), st));
    const BlockW w{m->wbase + m->wl.eqkv[seg], m->wbase + m->wl.ewo[seg], m->wbase + m->wl.egu[seg], m->wbase + m->wl.ewd[seg],
                   m->gain(m->wl.gm[seg])};
    return run_block(m, c, me, T, eh->n_qt, cf.n_layers + seg, w, c->xgh(), !with_head, m->exit_out_gain(seg), nullptr, false, max_ctx,
                     st);
}

// head `hi` (exit number, or n_exits for the final head) on the rows listed in dev_desc(di).head_*
int run_head(ee_model* m, ee_kv_cache* c, int di, int hi, int n_head, int mode, float threshold, hipStream_t st) {
    const ee_config& cf = m->cfg;
    const int d = cf.d_model, dt = cf.dtype;
    bool fin = hi >= cf.n_exits;
    SegDesc* dd = m->dev_desc(di);
    GemmCommon g{};
    g.dtype = dt;
    g.min_wgs = cf.gemm_min_workgroups;
    g.inv_d = 1.0f / (float)d;
    g.eps = cf.rms_eps;
    g.ssq_stride = c->ssq_stride;
    g.ssq_n = c->ssq_stride;
    g.T = n_head;
    void* a_rows = fin ? c->xg() : c->xgh();  // x.g of the gain this head reads first
    const SegDesc* hd = m->host_desc(di);
    if (!fin && m->exit_layer()) {  // run_exit_layer has left x'.g at the copies' slots
        dd = m->dev_desc(m->mlp_desc(di));
        hd = m->host_desc(m->mlp_desc(di));
        a_rows = c->xg();
    }
    if (!fin && m->exit_mlp()) {
        // The exit's MLP works on copies of the head rows, so that the backbone's rows stay as they are; its down
        // projection leaves x'.g (g: the exit's norm gain, or 1) in the first operand store at the copies' slots.
        const int me = m->mlp_desc(di);
        const SegDesc* eh = m->host_desc(me);
        if (eh->T != n_head || hd->n_head != n_head) return EE_ERR_STATE;
        SegDesc* ed = m->dev_desc(me);
        const int32_t* src = (const int32_t*)((char*)dd + offsetof(SegDesc, head_xrow));
        const int32_t* dst = (const int32_t*)((char*)ed + offsetof(SegDesc, xrow));
        HIPCHK(launch_copy_slots(dt, src, dst, n_head, d, c->x(), c->xgh(), c->xs_lo, c->ssq(), c->ssq_stride, st));
        const bool pk_d = dt == EE_BF16 && !gemm_rows_fit_lds(dt, n_head, d);
        const bool pk_F = dt == EE_BF16 && !gemm_rows_fit_lds(dt, n_head, cf.d_ff);
        if (pk_d) HIPCHK(launch_pack_rows(c->xgh(), c->xs_lo, d, dst, n_head, d, m->ws + m->wsl.xg_pk, m->lo_rows(d), st));
        g.desc = ed;
        g.desc_host = eh;
        EECHK(run_mlp(m, c, g, m->wbase + m->wl.egu[hi], m->wbase + m->wl.ewd[hi], c->xgh(), dst, pk_d, pk_F, m->exit_out_gain(hi),
                      nullptr, false, st));
        dd = ed;
        hd = eh;
        a_rows = c->xg();
    }
    g.desc = dd;
    g.desc_host = hd;
    g.W = m->wbase + (fin ? m->wl.wf : m->wl.we[hi]);
    g.N = cf.vocab;
    g.K = d;
    g.A = a_rows;
    g.a_lo = c->xs_lo;
    g.a_packed = 0;
    g.lda = d;
    g.arow = (const int32_t*)((char*)dd + offsetof(SegDesc, head_xrow));
    if (dt == EE_BF16 && !gemm_rows_fit_lds(dt, n_head, d)) {  // many rows: packed operands
        char* hp = m->ws + m->wsl.head_pk;
        HIPCHK(launch_pack_rows(g.A, g.a_lo, d, g.arow, n_head, d, hp, (size_t)64 * d, st));
        g.A = hp;
        g.a_lo = (size_t)64 * d;
        g.a_packed = 1;
    }
    g.ssq = (fin || m->exit_norm()) ? c->ssq() : nullptr;  // an exit without a norm reads x as it is
    float* logits = (m->dbg_logits && n_head <= m->dbg_rows) ? m->dbg_logits : nullptr;
    Timed t(m, EE_K_HEAD, st);
    m->head_tag = m->head_tag == 0x7fffffff ? 1 : m->head_tag + 1;
    HIPCHK(launch_gemm_head(g, (HeadPartial*)(m->ws + m->wsl.partials), (int32_t*)(m->ws + m->wsl.counters), logits, mode,
                            threshold, m->results_dev, m->head_tag, st));
    return EE_OK;
}

// Waits until the head evaluation launched last has written the results of the n_head rows listed in `hd`.
// The results are in host memory: polling their tags returns a few microseconds after the kernel's store,
// where a stream synchronisation takes tens of microseconds to wake the caller up.  The stream is queried
// every so often, so that a failed launch (or a drained stream) ends the wait.
int wait_head_results(ee_model* m, const SegDesc* hd, hipStream_t st) {
    const int tag = m->head_tag;
    const auto t0 = std::chrono::steady_clock::now();
    for (unsigned spins = 1;; ++spins) {
        bool all = true;
        for (int i = 0; i < hd->n_head && all; ++i)
            all = __atomic_load_n(&m->results[hd->head_slot[i]].pad, __ATOMIC_ACQUIRE) == tag;
        if (all) return EE_OK;
        if ((spins & 1023) == 0) {
            hipError_t q = hipStreamQuery(st);
            if (q == hipSuccess) {
                HIPCHK(hipStreamSynchronize(st));
                return EE_OK;
            }
            if (q != hipErrorNotReady) HIPCHK(q);
            // A step takes milliseconds; a stream that is still busy after this long will not finish.
            if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(m->head_wait_limit_s)) {
                g_last_hip = (int)hipErrorNotReady;
                return EE_ERR_HIP;
            }
        }
#if defined(__x86_64__)
        __builtin_ia32_pause();
#endif
    }
}

int ensure_blocks(ee_kv_cache* c, SeqState& s, int n_positions) {
    int need = (n_positions + c->BT - 1) / c->BT;
    if (need > c->geom.max_blocks_per_seq) return EE_ERR_RANGE;
    while ((int)s.blocks.size() < need) {
        if (c->free_blocks.empty()) return EE_ERR_NOMEM;
        s.blocks.push_back(c->free_blocks.back());
        c->free_blocks.pop_back();
    }
    return EE_OK;
}

void put_btab(const ee_model* m, const ee_kv_cache* c, int row, const SeqState& s) {
    int32_t* bt = m->host_btab() + (size_t)row * c->geom.max_blocks_per_seq;
    std::copy(s.blocks.begin(), s.blocks.end(), bt);
}

// What of the upload region a step needs: the descriptors of the model's segments, those of the exits' own rows (if
// the exits work on copies), and the block tables and token ids behind them.
void upload_ranges(const ee_model* m, uint32_t off16[3], uint32_t n16[3]) {
    const WorkspaceLayout& w = m->wsl;
    off16[0] = (uint32_t)((w.descs - w.upload) / 16);
    n16[0] = (uint32_t)((sizeof(SegDesc) * m->n_seg() + 15) / 16);
    off16[1] = (uint32_t)((w.descs - w.upload + sizeof(SegDesc) * (EE_MAX_EXITS + 1)) / 16);
    n16[1] = m->exit_block() ? (uint32_t)((sizeof(SegDesc) * m->cfg.n_exits + 15) / 16) : 0;
    off16[2] = (uint32_t)((w.btab - w.upload) / 16);
    n16[2] = (uint32_t)((w.upload + w.upload_bytes - w.btab + 15) / 16);
}

// Descriptors, block tables and token ids of the step: staging area -> workspace; with embed_rows > 0 the same launch
// looks up the rows of host_desc(0) in the embedding.
int upload(ee_model* m, hipStream_t st, int embed_rows = 0, ee_kv_cache* c = nullptr) {
    uint32_t off16[3], n16[3];
    upload_ranges(m, off16, n16);
    const SegDesc* d0 = m->host_desc(0);
    const SegDesc* d0_dev = (const SegDesc*)(m->pinned_dev + (m->wsl.descs - m->wsl.upload));
    HIPCHK(launch_step_begin(m->cfg.dtype, m->pinned_dev, m->ws + m->wsl.upload, off16, n16, embed_rows, m->host_tokens(), d0->xrow,
                             (const int32_t*)(m->pinned_dev + (m->wsl.tokens - m->wsl.upload)), d0_dev->xrow,
                             m->wbase + m->wl.embed, m->cfg.d_model, m->gain(m->wl.g1[0]), c ? c->x() : nullptr, c ? c->xg() : nullptr,
                             c ? c->xs_lo : 0, c ? c->ssq() : nullptr, c ? c->ssq_stride : 0, st));
    return EE_OK;
}

struct StepSeq {
    int seq, p;     // sequence id, position of the current token (or -1 for a flush)
    bool forced, active;
};

// rows of the active sequences for segment `seg`: positions [filled[seg], last] of each
void build_desc(const ee_model* m, const ee_kv_cache* c, SegDesc* d, const std::vector<StepSeq>& ss, int seg, bool with_head,
                float threshold, int* rows_out) {
    int T = 0, nqt = 0, nh = 0;
    for (size_t b = 0; b < ss.size(); ++b) {
        if (!ss[b].active) continue;
        const SeqState& s = c->seqs[ss[b].seq];
        int lo, hi;  // inclusive
        plan::rows(s.filled.data(), (int)s.filled.size(), seg, ss[b].p, c->refeed != 0, &lo, &hi);
        int first = T;
        for (int pos = lo; pos <= hi; ++pos, ++T) {
            if (T >= EE_MAX_ROWS) { *rows_out = EE_MAX_ROWS + 1; return; }
            d->xrow[T] = c->slot_of(ss[b].seq, pos);
            if (seg == 0) m->host_tokens()[T] = s.tokring[pos % c->S];  // rows that start at the embedding
            d->pos[T] = pos;
            d->kvblk[T] = s.blocks[pos / c->BT];
            d->rseq[T] = (int)b;
        }
        for (int r = first; r < T; r += 16) {
            d->qt_row0[nqt] = r;
            d->qt_nq[nqt] = std::min(16, T - r);
            d->qt_pos0[nqt] = d->pos[r];
            d->qt_seq[nqt] = (int)b;
            ++nqt;
        }
        bool is_final = seg == m->n_seg() - 1;
        if (with_head && ss[b].p >= 0 && T > first && (is_final || (!ss[b].forced && threshold < 1.0f))) {
            d->head_xrow[nh] = c->slot_of(ss[b].seq, ss[b].p);
            d->head_slot[nh] = seg * EE_MAX_SEQS + (int)b;
            ++nh;
        }
    }
    // Query tiles in order of falling context length: the attention workgroups of a launch are handed out in tile
    // order, and the longest ones must not be the last to start (the rows themselves stay where they are).
    {
        struct Tile {
            int32_t row0, nq, pos0, seq;
        };
        Tile tiles[EE_MAX_ROWS];
        for (int i = 0; i < nqt; ++i) tiles[i] = Tile{d->qt_row0[i], d->qt_nq[i], d->qt_pos0[i], d->qt_seq[i]};
        std::stable_sort(tiles, tiles + nqt, [](const Tile& a, const Tile& b) { return a.pos0 + a.nq > b.pos0 + b.nq; });
        for (int i = 0; i < nqt; ++i) {
            d->qt_row0[i] = tiles[i].row0;
            d->qt_nq[i] = tiles[i].nq;
            d->qt_pos0[i] = tiles[i].pos0;
            d->qt_seq[i] = tiles[i].seq;
        }
    }
    for (int i = 0; i < nqt; ++i)
        for (int q = 0; q < d->qt_nq[i]; ++q) d->row_qt[d->qt_row0[i] + q] = i * 16 + q;
    d->T = T;
    d->n_qt = nqt;
    d->n_head = nh;
    d->pad = 0;
    fill_mlp_desc(m, c, seg);
    *rows_out = T;
}

int max_ctx_of(const ee_kv_cache* c, const std::vector<StepSeq>& ss) {
    int mx = 1;
    for (auto& q : ss) mx = std::max(mx, (q.p >= 0 ? q.p : c->seqs[q.seq].filled[0] - 1) + 1);
    return mx;
}

// Work that an earlier decode step left running on another stream (see ee_model::spec_ev) is waited for first.
int settle(ee_model* m, hipStream_t st) {
    if (m->spec_recorded && st != m->spec_stream) HIPCHK(hipStreamWaitEvent(st, m->spec_ev, 0));
    return EE_OK;
}

// Common engine of decode and flush.  For a flush p = -1 everywhere and no head runs.
int run_step(ee_model* m, ee_kv_cache* c, std::vector<StepSeq>& ss, float threshold, bool decode, int32_t* next_token,
             int32_t* exit_layer, float* conf, hipStream_t st) {
    const int n_seg = m->n_seg();
    EECHK(settle(m, st));
    if (decode) m->step_tag0 = m->head_tag;
    for (size_t b = 0; b < ss.size(); ++b) put_btab(m, c, (int)b, c->seqs[ss[b].seq]);
    int max_ctx = max_ctx_of(c, ss);
    std::vector<int> rows(n_seg, 0);
    auto rebuild = [&](int from) -> int {
        for (int s = from; s < n_seg; ++s) {
            build_desc(m, c, m->host_desc(s), ss, s, decode, threshold, &rows[s]);
            if (rows[s] > m->max_rows) return EE_ERR_NOMEM;
        }
        // (the first upload of a step also looks up the rows that start at the embedding)
        const bool embed = from == 0 && (decode || c->refeed) && m->host_desc(0)->T > 0;
        return upload(m, st, embed ? m->host_desc(0)->T : 0, c);
    };
    EECHK(rebuild(0));
    int n_active = (int)ss.size();
    Pipeline& pp = c->pipe;
    int spec_seg = -1, spec_ns = 0;  // segment whose first layer's KV write and attention are already enqueued
    for (int s = 0; s < n_seg && n_active > 0; ++s) {
        const SegDesc* hd = m->host_desc(s);
        if (hd->T > 0) {
            // pipeline mode: the stage's previous token may still be on the other stream (segment 0 only ever runs here)
            if (pp.on && s > 0 && pp.last_ev[s] >= 0 && pp.last_stream[s] != st)
                HIPCHK(hipStreamWaitEvent(st, pp.pool[pp.last_ev[s]], 0));
            EECHK(run_layers(m, c, s, hd->T, hd->n_qt, m->seg_begin(s), m->seg_end(s), max_ctx, st, spec_seg == s ? BLOCK_REST : BLOCK_ALL,
                             &spec_ns));
            if (m->exit_layer() && s < m->cfg.n_exits)
                EECHK(run_exit_layer(m, c, s, (const int32_t*)((char*)m->dev_desc(s) + offsetof(SegDesc, xrow)), decode && hd->n_head > 0,
                                     max_ctx, st));
            if (pp.on && s > 0) {
                const int e = pp.next_ev++ % Pipeline::POOL;
                HIPCHK(hipEventRecord(pp.pool[e], st));
                pp.last_ev[s] = e;
                pp.last_stream[s] = st;
            }
        }
        bool is_final = s == n_seg - 1;
        if (decode && hd->n_head > 0) {
            EECHK(run_head(m, c, s, s, hd->n_head, is_final ? HEAD_EMIT : HEAD_RULE, threshold, st));
            // One sequence: either it leaves here or the next segment runs on the rows already described.  Its first
            // layer's KV write and attention are enqueued before the host knows which, so that the GPU does not stand
            // idle while the result travels and the launches follow.  They change nothing a token that leaves depends
            // on: K and V of rows whose watermark for that segment stays where it was (the pass that does advance it
            // writes them again), and the q, attention and partial buffers of the workspace.  The residual stream is
            // first touched by the O projection, which waits for the decision.
            if (!is_final && ss.size() == 1 && !pp.on) {
                const SegDesc* nd = m->host_desc(s + 1);
                const int dt = m->cfg.dtype;
                if (nd->T > 0 && (dt != EE_BF16 || gemm_rows_fit_lds(dt, nd->T, m->cfg.d_model))) {
                    EECHK(run_layers(m, c, s + 1, nd->T, nd->n_qt, m->seg_begin(s + 1), m->seg_end(s + 1), max_ctx, st, BLOCK_FRONT, &spec_ns));
                    spec_seg = s + 1;
                    HIPCHK(hipEventRecord(m->spec_ev, st));
                    m->spec_stream = st;
                    m->spec_recorded = true;
                    c->spec_used = true;
                }
            }
            EECHK(wait_head_results(m, hd, st));
            int fired_now = 0;
            for (int i = 0; i < hd->n_head; ++i) {
                int slot = hd->head_slot[i];
                int b = slot - s * EE_MAX_SEQS;
                const HeadResult& r = m->results[slot];
                if (r.fired) {
                    next_token[b] = r.token;
                    exit_layer[b] = m->seg_end(s);
                    if (conf) conf[b] = r.conf;
                    ss[b].active = false;
                    SeqState& sq = c->seqs[ss[b].seq];
                    plan::commit(sq.filled.data(), s, ss[b].p);
                    ++fired_now;
                }
            }
            n_active -= fired_now;
            if (fired_now && n_active > 0 && !is_final) EECHK(rebuild(s + 1));
        }
        if (is_final) {
            if (!decode) {
                for (auto& q : ss) {
                    SeqState& sq = c->seqs[q.seq];
                    plan::flushed(sq.filled.data(), n_seg);
                }
                if (!pp.on) HIPCHK(hipStreamSynchronize(st));  // (a pipelined fill is waited for through its events)
            }
        }
    }
    return EE_OK;
}

// Pipeline mode, after a decode step: the tokens that left at an exit go through their remaining segments on the
// fill stream (no head, nothing emitted), in that stream's own workspace; the call only enqueues.  Their watermarks
// advance now: every later pass over those segments is ordered behind this one by the per-segment events.
int pipeline_fill(ee_model* m, ee_kv_cache* c, const std::vector<StepSeq>& step) {
    Pipeline& pp = c->pipe;
    std::vector<StepSeq> fs;
    for (const StepSeq& q : step)
        if (c->n_pending(c->seqs[q.seq]) > 0) fs.push_back(StepSeq{q.seq, -1, true, true});
    if (fs.empty()) return EE_OK;
    const int slot = pp.next_slot;
    pp.next_slot = (slot + 1) % Pipeline::RING;
    if (pp.slot_used[slot]) HIPCHK(hipEventSynchronize(pp.slot_done[slot]));  // its descriptors have been read
    char *ws = m->ws, *pin = m->pinned, *pin_dev = m->pinned_dev;
    m->ws = pp.ws;
    m->pinned = pp.pinned + (size_t)slot * pp.slot_bytes;
    m->pinned_dev = pp.pinned_dev + (size_t)slot * pp.slot_bytes;
    int rc = run_step(m, c, fs, 1.0f, false, nullptr, nullptr, nullptr, pp.stream);
    m->ws = ws;
    m->pinned = pin;
    m->pinned_dev = pin_dev;
    EECHK(rc);
    HIPCHK(hipEventRecord(pp.slot_done[slot], pp.stream));
    pp.slot_used[slot] = true;
    return EE_OK;
}

int pipeline_drain(ee_kv_cache* c) {
    if (c->pipe.on) HIPCHK(hipStreamSynchronize(c->pipe.stream));
    return EE_OK;
}

// ---- prompt phase through the GEMM path: whole passes of up to pf_rows positions, every projection one
// matrix-core GEMM over all rows, causal attention over the pass and the cache before it.  The last
// position's residual row is handed to the decode-side store after each segment, where the usual heads
// decide the first token.  score_tok / score_conf (host, [n_seg][n_tokens], optional): every head on
// every position.
int prefill_large(ee_model* m, ee_kv_cache* c, int seq, const int32_t* tokens, int n_tokens, float threshold, int32_t* score_tok,
                  float* score_conf, float* score_nll, hipStream_t st) {
    const ee_config& cf = m->cfg;
    const WorkspaceLayout& w = m->wsl;
    const int d = cf.d_model, F = cf.d_ff, V = cf.vocab, n_seg = m->n_seg();
    const size_t Mp = w.pf_rows;
    const int ssq_n = (d + 255) / 256;
    SeqState& s = c->seqs[seq];
    char* ws = m->ws;
    float* x = (float*)(ws + w.pf_x);
    char *xg_hi = ws + w.pf_xg, *xg_lo = xg_hi + Mp * d * 2;
    char *xgh_hi = ws + w.pf_xgh, *xgh_lo = xgh_hi + Mp * d * 2;
    char *q_hi = ws + w.pf_q, *q_lo = q_hi + Mp * d * 2;
    char *at_hi = ws + w.pf_attn, *at_lo = at_hi + Mp * d * 2;
    char *ac_hi = ws + w.pf_act, *ac_lo = ac_hi + Mp * F * 2;
    float* ssq = (float*)(ws + w.pf_ssq);
    const int slot = c->slot_of(seq, n_tokens - 1);
    put_btab(m, c, 0, s);
    for (int i = 0; i < n_seg; ++i) {  // one descriptor per head so that each writes its own result slot
        SegDesc* di = m->host_desc(i);
        di->T = 0;
        di->n_qt = 0;
        di->n_head = 1;
        di->head_xrow[0] = slot;
        di->head_slot[0] = i * EE_MAX_SEQS;
        fill_mlp_desc(m, c, i);
        if (m->exit_layer() && i < cf.n_exits) {  // the exit's layer runs on a copy of the last position's row
            SegDesc* e = m->host_desc(m->mlp_desc(i));
            e->T = e->n_qt = e->n_head = 1;
            e->pad = 0;
            e->xrow[0] = e->head_xrow[0] = c->exit_slot(0);
            e->pos[0] = e->qt_pos0[0] = n_tokens - 1;
            e->kvblk[0] = s.blocks[(n_tokens - 1) / c->BT];
            e->rseq[0] = e->row_qt[0] = e->qt_row0[0] = e->qt_seq[0] = 0;
            e->qt_nq[0] = 1;
            e->head_slot[0] = i * EE_MAX_SEQS;
        }
    }
    EECHK(upload(m, st));
    const int32_t* bt = m->dev_btab();
    PfGemm g{};
    g.inv_d = 1.0f / (float)d;
    g.eps = cf.rms_eps;
    g.ssq_n = ssq_n;
    for (int p0 = 0; p0 < n_tokens; p0 += (int)Mp) {
        const int M = std::min((int)Mp, n_tokens - p0);
        const bool last = p0 + M == n_tokens;
        g.M = M;
        std::memcpy(m->pf_host_tokens, tokens + p0, (size_t)M * 4);
        HIPCHK(hipMemcpyAsync(ws + w.pf_tokens, m->pf_host_tokens, (size_t)M * 4, hipMemcpyHostToDevice, st));
        if (score_nll) {  // the token that follows each position (none after the last one of the prompt)
            int32_t* tg = m->pf_host_tokens + Mp;
            for (int r = 0; r < M; ++r) tg[r] = p0 + r + 1 < n_tokens ? tokens[p0 + r + 1] : -1;
            HIPCHK(hipMemcpyAsync(ws + w.pf_tgt, tg, (size_t)M * 4, hipMemcpyHostToDevice, st));
        }
        HIPCHK(launch_pf_embed(m->wbase + m->wl.embed, (const int32_t*)(ws + w.pf_tokens), M, d, m->gain(m->wl.g1[0]), x, xg_hi, xg_lo, ssq,
                               ssq_n, st));
        for (int sgi = 0; sgi < n_seg; ++sgi) {
            const bool fin = sgi == n_seg - 1;
            for (int l = m->seg_begin(sgi); l < m->seg_end(sgi); ++l) {
                g.W = m->wbase + m->wl.qkv[l];
                g.N = 3 * d;
                g.K = d;
                g.A_hi = xg_hi;
                g.A_lo = xg_lo;
                g.ssq = ssq;
                {
                    Timed t(m, EE_K_QKV, st);
                    HIPCHK(launch_pf_qkv(g, q_hi, q_lo, (const float*)(m->wbase + m->wl.rope), c->geom, l, bt, p0, st));
                }
                {
                    Timed t(m, EE_K_ATTN, st);
                    HIPCHK(launch_pf_attention(q_hi, q_lo, at_hi, at_lo, c->geom, l, bt, p0, M, d, st));
                }
                g.W = m->wbase + m->wl.wo[l];
                g.N = d;
                g.A_hi = at_hi;
                g.A_lo = at_lo;
                g.ssq = nullptr;
                {
                    Timed t(m, EE_K_OPROJ, st);
                    HIPCHK(launch_pf_resid(g, x, xg_hi, xg_lo, nullptr, nullptr, m->gain(m->wl.g2[l]), nullptr, ssq, ssq_n, st));
                }
                g.W = m->wbase + m->wl.gu[l];
                g.N = 2 * F;
                g.A_hi = xg_hi;
                g.A_lo = xg_lo;
                g.ssq = ssq;
                {
                    Timed t(m, EE_K_SWIGLU, st);
                    HIPCHK(launch_pf_swiglu(g, ac_hi, ac_lo, F, st));
                }
                g.W = m->wbase + m->wl.wd[l];
                g.N = d;
                g.K = F;
                g.A_hi = ac_hi;
                g.A_lo = ac_lo;
                g.ssq = nullptr;
                const float* g_next = (l + 1 < cf.n_layers) ? m->gain(m->wl.g1[l + 1]) : m->gain(m->wl.gf);
                const float* g_head = (!fin && l + 1 == m->seg_end(sgi)) ? m->exit_in_gain(sgi) : nullptr;
                {
                    Timed t(m, EE_K_DOWN, st);
                    HIPCHK(launch_pf_resid(g, x, xg_hi, xg_lo, g_head ? xgh_hi : nullptr, g_head ? xgh_lo : nullptr, g_next, g_head, ssq,
                                           ssq_n, st));
                }
            }
            if (!fin && m->exit_layer()) {
                // every position of the pass leaves its K and V in the exit's own layer (the q it also forms is not used)
                g.W = m->wbase + m->wl.eqkv[sgi];
                g.N = 3 * d;
                g.K = d;
                g.A_hi = xgh_hi;
                g.A_lo = xgh_lo;
                g.ssq = ssq;
                Timed t(m, EE_K_QKV, st);
                HIPCHK(launch_pf_qkv(g, q_hi, q_lo, (const float*)(m->wbase + m->wl.rope), c->geom, cf.n_layers + sgi, bt, p0, st));
            }
            if (score_tok || score_conf || score_nll) {  // this segment's head on every position of the pass
                const float* head_ssq = ssq;
                const char *ha_hi = fin ? xg_hi : xgh_hi, *ha_lo = fin ? xg_lo : xgh_lo;
                if (!fin && m->exit_mlp()) {
                    // The exit's MLP on every position, on a copy of the residual rows: the buffers of q and of the
                    // attention output are free between layers and take the copy and its operand x'.g.
                    float* xe = (float*)q_hi;
                    float* ssq_e = (float*)(ws + w.pf_ssqe);
                    HIPCHK(hipMemcpyAsync(xe, x, (size_t)M * d * 4, hipMemcpyDeviceToDevice, st));
                    g.W = m->wbase + m->wl.egu[sgi];
                    g.N = 2 * F;
                    g.K = d;
                    g.A_hi = xgh_hi;
                    g.A_lo = xgh_lo;
                    g.ssq = ssq;
                    {
                        Timed t(m, EE_K_SWIGLU, st);
                        HIPCHK(launch_pf_swiglu(g, ac_hi, ac_lo, F, st));
                    }
                    g.W = m->wbase + m->wl.ewd[sgi];
                    g.N = d;
                    g.K = F;
                    g.A_hi = ac_hi;
                    g.A_lo = ac_lo;
                    g.ssq = nullptr;
                    {
                        Timed t(m, EE_K_DOWN, st);
                        HIPCHK(launch_pf_resid(g, xe, at_hi, at_lo, nullptr, nullptr, m->exit_out_gain(sgi), nullptr, ssq_e, ssq_n, st));
                    }
                    ha_hi = at_hi;
                    ha_lo = at_lo;
                    head_ssq = ssq_e;
                }
                g.W = m->wbase + (fin ? m->wl.wf : m->wl.we[sgi]);
                g.N = V;
                g.K = d;
                g.A_hi = ha_hi;
                g.A_lo = ha_lo;
                g.ssq = (fin || m->exit_norm()) ? head_ssq : nullptr;  // an exit without a norm reads x as it is
                {
                    Timed t(m, EE_K_HEAD, st);
                    HIPCHK(launch_pf_head(g, (HeadPartial*)(ws + w.pf_partials), (int32_t*)(ws + w.pf_tok), (float*)(ws + w.pf_conf),
                                          (const int32_t*)(ws + w.pf_tgt), (float*)(ws + w.pf_zt), score_nll ? (float*)(ws + w.pf_nll) : nullptr,
                                          cf.scored_head_terms == 2, st));
                }
                if (score_tok)
                    HIPCHK(hipMemcpyAsync(score_tok + (size_t)sgi * n_tokens + p0, ws + w.pf_tok, (size_t)M * 4, hipMemcpyDeviceToHost, st));
                if (score_conf)
                    HIPCHK(hipMemcpyAsync(score_conf + (size_t)sgi * n_tokens + p0, ws + w.pf_conf, (size_t)M * 4, hipMemcpyDeviceToHost, st));
                if (score_nll)
                    HIPCHK(hipMemcpyAsync(score_nll + (size_t)sgi * n_tokens + p0, ws + w.pf_nll, (size_t)M * 4, hipMemcpyDeviceToHost, st));
            }
            if (last && (fin || threshold < 1.0f)) {
                const int l_end = m->seg_end(sgi);
                const float* g_a = fin ? m->gain(m->wl.gf) : m->gain(m->wl.g1[l_end]);
                const float* g_b = fin ? nullptr : m->exit_in_gain(sgi);
                const size_t es = 2;
                HIPCHK(launch_pf_export_row(x + (size_t)(M - 1) * d, d, g_a, g_b, c->x() + (size_t)slot * d,
                                            (char*)c->xg() + (size_t)slot * d * es, (char*)c->xgh() + (size_t)slot * d * es, c->xs_lo,
                                            c->ssq() + (size_t)slot * c->ssq_stride, c->ssq_stride, st));
                if (!fin && m->exit_layer())
                    EECHK(run_exit_layer(m, c, sgi, (const int32_t*)((char*)m->dev_desc(sgi) + offsetof(SegDesc, head_xrow)), true,
                                         n_tokens, st));
                EECHK(run_head(m, c, sgi, sgi, 1, fin ? HEAD_EMIT : HEAD_RULE, threshold, st));
            }
        }
        HIPCHK(hipStreamSynchronize(st));  // the pinned token staging is rewritten by the next pass
    }
    return EE_OK;
}

}  // namespace

extern "C" {

const char* ee_strerror(int code) {
    switch (code) {
        case EE_OK: return "ok";
        case EE_ERR_CONFIG: return "bad or unsupported configuration";
        case EE_ERR_NOMEM: return "buffer too small or KV block pool exhausted";
        case EE_ERR_RANGE: return "token, sequence id or position out of range";
        case EE_ERR_STATE: return "arguments disagree with the cache state, or tensors missing";
        case EE_ERR_IO: return "weight file unreadable or malformed";
        case EE_ERR_HIP: return "HIP call failed";
        case EE_ERR_ARG: return "null or misaligned pointer, or bad count";
    }
    return "unknown error";
}

int ee_last_hip_error(void) { return g_last_hip; }

int ee_model_bytes(const ee_config* cfg, int max_rows, int max_seqs, size_t* weight_bytes, size_t* workspace_bytes) {
    if (!cfg) return EE_ERR_ARG;
    EECHK(check_config(*cfg));
    if (max_rows < 1 || max_rows > EE_MAX_ROWS || max_seqs < 1 || max_seqs > EE_MAX_SEQS) return EE_ERR_CONFIG;
    if (weight_bytes) *weight_bytes = weight_layout(*cfg).total;
    if (workspace_bytes) *workspace_bytes = workspace_layout(*cfg, max_rows, max_seqs).total;
    return EE_OK;
}

int ee_model_create(const ee_config* cfg, void* dev_weights, size_t weight_bytes, void* dev_workspace,
                    size_t workspace_bytes, int max_rows, int max_seqs, void* stream, ee_model** out) {
    if (!cfg || !dev_weights || !dev_workspace || !out) return EE_ERR_ARG;
    if (((uintptr_t)dev_weights | (uintptr_t)dev_workspace) & 255) return EE_ERR_ARG;
    size_t wb, sb;
    EECHK(ee_model_bytes(cfg, max_rows, max_seqs, &wb, &sb));
    if (weight_bytes < wb || workspace_bytes < sb) return EE_ERR_NOMEM;
    ee_model* m = new (std::nothrow) ee_model();
    if (!m) return EE_ERR_NOMEM;
    m->cfg = *cfg;
    m->max_rows = max_rows;
    m->max_seqs = max_seqs;
    m->wbase = (char*)dev_weights;
    m->ws = (char*)dev_workspace;
    m->wl = weight_layout(*cfg);
    m->wsl = workspace_layout(*cfg, max_rows, max_seqs);
    m->have.assign(m->n_tensors(), 0);
    m->n_missing = m->n_tensors();
    for (int kind = 0; kind < EE_T_KINDS; ++kind)
        for (int idx = 0; !m->applicable(kind) && m->tensor_slot(kind, idx) >= 0; ++idx) {
            m->have[m->tensor_slot(kind, idx)] = 1;
            --m->n_missing;
        }
    m->dbg_logits = nullptr;
    m->dbg_rows = 0;
    size_t res_bytes = align_up(sizeof(HeadResult) * EE_MAX_SEQS * (EE_MAX_EXITS + 1)) + (size_t)m->wsl.pf_rows * 8;  // tokens and next-token targets of a pass
    hipError_t e = hipHostMalloc((void**)&m->pinned, align_up(m->wsl.upload_bytes) + res_bytes, hipHostMallocMapped);
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        delete m;
        return EE_ERR_HIP;
    }
    std::memset(m->pinned, 0, align_up(m->wsl.upload_bytes) + res_bytes);
    m->results = (HeadResult*)(m->pinned + align_up(m->wsl.upload_bytes));
    m->pf_host_tokens = (int32_t*)((char*)m->results + align_up(sizeof(HeadResult) * EE_MAX_SEQS * (EE_MAX_EXITS + 1)));
    hipStream_t st = (hipStream_t)stream;
    int rc = EE_OK;
    do {
        if ((e = hipHostGetDevicePointer((void**)&m->results_dev, m->results, 0)) != hipSuccess) break;
        if ((e = hipHostGetDevicePointer((void**)&m->pinned_dev, m->pinned, 0)) != hipSuccess) break;
        if ((e = hipEventCreateWithFlags(&m->spec_ev, hipEventDisableTiming)) != hipSuccess) break;  // (no step creates anything)
        if ((e = hipMemsetAsync(m->ws + m->wsl.counters, 0, 256 * 4, st)) != hipSuccess) break;
        if ((e = launch_fill_f32((float*)(m->wbase + m->wl.ones), 1.0f, (size_t)cfg->d_model, st)) != hipSuccess) break;
        if (m->wsl.pf_rows && (e = hipMemsetAsync(m->ws + m->wsl.pf_begin, 0, m->wsl.total - m->wsl.pf_begin, st)) != hipSuccess) break;
        e = launch_rope_table((float*)(m->wbase + m->wl.rope), cfg->max_positions, cfg->head_dim, cfg->rope_base, st);
    } while (0);
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        rc = EE_ERR_HIP;
        if (m->spec_ev) (void)hipEventDestroy(m->spec_ev);
        (void)hipHostFree(m->pinned);
        delete m;
        return rc;
    }
    *out = m;
    return EE_OK;
}

int ee_model_set_tensor(ee_model* m, int kind, int index, const void* dev_src, size_t n_elems, void* stream) {
    if (!m || !dev_src) return EE_ERR_ARG;
    int slot = m->tensor_slot(kind, index);
    if (slot < 0) return EE_ERR_RANGE;
    if (!m->applicable(kind)) return EE_ERR_CONFIG;
    const ee_config& c = m->cfg;
    const size_t d = c.d_model, F = c.d_ff, V = c.vocab, es = esize(c.dtype);
    const int dt = c.dtype, hd = c.head_dim;
    hipStream_t st = (hipStream_t)stream;
    EECHK(settle(m, st));
    auto gain = [&](size_t off) -> int {
        if (n_elems != d) return EE_ERR_ARG;
        HIPCHK(hipMemcpyAsync(m->wbase + off, dev_src, d * 4, hipMemcpyDeviceToDevice, st));
        return EE_OK;
    };
    auto mat = [&](size_t off, size_t rows, size_t K, int mode) -> int {
        if (n_elems != rows * K) return EE_ERR_ARG;
        HIPCHK(launch_pack(dt, dev_src, m->wbase + off, (int)rows, (int)K, mode, hd, st));
        return EE_OK;
    };
    int rc;
    switch (kind) {
        case EE_T_EMBED:
            if (n_elems != V * d) return EE_ERR_ARG;
            HIPCHK(hipMemcpyAsync(m->wbase + m->wl.embed, dev_src, V * d * es, hipMemcpyDeviceToDevice, st));
            rc = m->tied() ? mat(m->wl.wf, V, d, PACK_PLAIN) : EE_OK;  // tied: also every head's matrix
            break;
        case EE_T_ATTN_NORM: rc = gain(m->wl.g1[index]); break;
        case EE_T_MLP_NORM: rc = gain(m->wl.g2[index]); break;
        case EE_T_EXIT_NORM: rc = gain(m->wl.ge[index]); break;
        case EE_T_FINAL_NORM: rc = gain(m->wl.gf); break;
        case EE_T_WQ: rc = mat(m->wl.qkv[index], d, d, PACK_ROTARY); break;
        case EE_T_WK: rc = mat(m->wl.qkv[index] + d * d * es, d, d, PACK_ROTARY); break;
        case EE_T_WV: rc = mat(m->wl.qkv[index] + 2 * d * d * es, d, d, PACK_ROTARY); break;
        case EE_T_WO: rc = mat(m->wl.wo[index], d, d, PACK_PLAIN); break;
        case EE_T_WG: rc = mat(m->wl.gu[index], F, d, PACK_GATE); break;
        case EE_T_WU: rc = mat(m->wl.gu[index], F, d, PACK_UP); break;
        case EE_T_WD: rc = mat(m->wl.wd[index], d, F, PACK_PLAIN); break;
        case EE_T_EXIT_HEAD: rc = mat(m->wl.we[index], V, d, PACK_PLAIN); break;
        case EE_T_FINAL_HEAD: rc = mat(m->wl.wf, V, d, PACK_PLAIN); break;
        case EE_T_EXIT_MLP_NORM: rc = gain(m->wl.gm[index]); break;
        case EE_T_EXIT_WG: rc = mat(m->wl.egu[index], F, d, PACK_GATE); break;
        case EE_T_EXIT_WU: rc = mat(m->wl.egu[index], F, d, PACK_UP); break;
        case EE_T_EXIT_WD: rc = mat(m->wl.ewd[index], d, F, PACK_PLAIN); break;
        case EE_T_EXIT_ATTN_NORM: rc = gain(m->wl.ga[index]); break;
        case EE_T_EXIT_WQ: rc = mat(m->wl.eqkv[index], d, d, PACK_ROTARY); break;
        case EE_T_EXIT_WK: rc = mat(m->wl.eqkv[index] + d * d * es, d, d, PACK_ROTARY); break;
        case EE_T_EXIT_WV: rc = mat(m->wl.eqkv[index] + 2 * d * d * es, d, d, PACK_ROTARY); break;
        case EE_T_EXIT_WO: rc = mat(m->wl.ewo[index], d, d, PACK_PLAIN); break;
        default: return EE_ERR_RANGE;
    }
    if (rc != EE_OK) return rc;
    if (!m->have[slot]) {
        m->have[slot] = 1;
        --m->n_missing;
    }
    return EE_OK;
}

int ee_model_load(const ee_config* cfg, const char* weights_path, void* dev_weights, size_t weight_bytes,
                  void* dev_workspace, size_t workspace_bytes, int max_rows, int max_seqs, void* dev_staging,
                  size_t staging_bytes, void* stream, ee_model** out) {
    if (!cfg || !weights_path || !dev_staging || !out) return EE_ERR_ARG;
    FILE* f = std::fopen(weights_path, "rb");
    if (!f) return EE_ERR_IO;
    char magic[8];
    ee_config fc;
    std::memset(&fc, 0, sizeof fc);
    bool ok = std::fread(magic, 1, 8, f) == 8;
    // "EEWT0001": the config without exit_flags (the default exit structure); "EEWT0002": with it
    const bool v2 = ok && std::memcmp(magic, "EEWT0002", 8) == 0;
    ok = ok && (v2 || std::memcmp(magic, "EEWT0001", 8) == 0);
    ok = ok && std::fread(&fc, v2 ? offsetof(ee_config, prefill_rows) : offsetof(ee_config, exit_flags), 1, f) == 1;
    if (!ok || fc.exit_flags != cfg->exit_flags) {
        std::fclose(f);
        return EE_ERR_IO;
    }
    if (fc.n_layers != cfg->n_layers || fc.d_model != cfg->d_model || fc.n_heads != cfg->n_heads || fc.d_ff != cfg->d_ff ||
        fc.vocab != cfg->vocab || fc.dtype != cfg->dtype || fc.n_exits != cfg->n_exits) {
        std::fclose(f);
        return EE_ERR_IO;
    }
    ee_model* m = nullptr;
    int rc = ee_model_create(cfg, dev_weights, weight_bytes, dev_workspace, workspace_bytes, max_rows, max_seqs, stream, &m);
    if (rc != EE_OK) {
        std::fclose(f);
        return rc;
    }
    const size_t d = cfg->d_model, F = cfg->d_ff, V = cfg->vocab, es = esize(cfg->dtype);
    const size_t chunk = 32u << 20;
    char* host = nullptr;
    hipError_t e = hipHostMalloc((void**)&host, chunk, hipHostMallocDefault);
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        std::fclose(f);
        ee_model_free(m);
        return EE_ERR_HIP;
    }
    hipStream_t st = (hipStream_t)stream;
    auto one = [&](int kind, int index, size_t n, size_t esz) -> int {
        size_t bytes = n * esz;
        if (bytes > staging_bytes) return EE_ERR_NOMEM;
        for (size_t o = 0; o < bytes; o += chunk) {
            size_t nb = std::min(chunk, bytes - o);
            if (std::fread(host, 1, nb, f) != nb) return EE_ERR_IO;
            HIPCHK(hipMemcpyAsync((char*)dev_staging + o, host, nb, hipMemcpyHostToDevice, st));
            HIPCHK(hipStreamSynchronize(st));
        }
        EECHK(ee_model_set_tensor(m, kind, index, dev_staging, n, stream));
        HIPCHK(hipStreamSynchronize(st));
        return EE_OK;
    };
    rc = one(EE_T_EMBED, 0, V * d, es);
    for (int l = 0; rc == EE_OK && l < cfg->n_layers; ++l) {
        const int kinds[] = {EE_T_ATTN_NORM, EE_T_WQ, EE_T_WK, EE_T_WV, EE_T_WO, EE_T_MLP_NORM, EE_T_WG, EE_T_WU, EE_T_WD};
        const size_t ns[] = {d, d * d, d * d, d * d, d * d, d, F * d, F * d, d * F};
        for (int j = 0; rc == EE_OK && j < 9; ++j)
            rc = one(kinds[j], l, ns[j], (kinds[j] == EE_T_ATTN_NORM || kinds[j] == EE_T_MLP_NORM) ? 4 : es);
    }
    for (int i = 0; rc == EE_OK && i < cfg->n_exits; ++i) {
        if (m->exit_layer()) {
            rc = one(EE_T_EXIT_ATTN_NORM, i, d, 4);
            for (int k : {EE_T_EXIT_WQ, EE_T_EXIT_WK, EE_T_EXIT_WV, EE_T_EXIT_WO})
                if (rc == EE_OK) rc = one(k, i, d * d, es);
        }
        if (rc == EE_OK && m->exit_block()) {
            rc = one(EE_T_EXIT_MLP_NORM, i, d, 4);
            if (rc == EE_OK) rc = one(EE_T_EXIT_WG, i, F * d, es);
            if (rc == EE_OK) rc = one(EE_T_EXIT_WU, i, F * d, es);
            if (rc == EE_OK) rc = one(EE_T_EXIT_WD, i, d * F, es);
        }
        if (rc == EE_OK && m->exit_norm()) rc = one(EE_T_EXIT_NORM, i, d, 4);
        if (rc == EE_OK && !m->tied()) rc = one(EE_T_EXIT_HEAD, i, V * d, es);
    }
    if (rc == EE_OK) rc = one(EE_T_FINAL_NORM, 0, d, 4);
    if (rc == EE_OK && !m->tied()) rc = one(EE_T_FINAL_HEAD, 0, V * d, es);
    std::fclose(f);
    (void)hipHostFree(host);
    if (rc != EE_OK) {
        ee_model_free(m);
        return rc;
    }
    *out = m;
    return EE_OK;
}

int ee_profile_begin(ee_model* m, int kernel, int max_launches) {
    if (!m || kernel < 0 || kernel >= EE_K_KINDS || max_launches < 1 || max_launches > (1 << 20)) return EE_ERR_ARG;
    // A fresh event costs several microseconds the first time it is recorded: new events are recorded once here, so
    // that the launches they are attached to later are not slowed down by it.
    bool fresh = false;
    while (m->prof_ev.size() < (size_t)max_launches * 2) {
        hipEvent_t e;
        HIPCHK(hipEventCreate(&e));
        m->prof_ev.push_back(e);
        HIPCHK(hipEventRecord(e, nullptr));
        fresh = true;
    }
    if (fresh) HIPCHK(hipStreamSynchronize(nullptr));
    m->prof_used = 0;
    m->prof_seen = 0;
    m->prof_kernel = kernel;
    return EE_OK;
}

int ee_profile_every(ee_model* m, int every) {
    if (!m || every < 1 || m->prof_kernel >= 0) return EE_ERR_ARG;
    m->prof_every = every;
    return EE_OK;
}

int ee_profile_end(ee_model* m, int32_t* n_launches, float* total_ms) {
    if (!m || !n_launches || !total_ms) return EE_ERR_ARG;
    m->prof_kernel = -1;
    float tot = 0.f;
    for (size_t i = 0; i + 1 < m->prof_used; i += 2) {
        HIPCHK(hipEventSynchronize(m->prof_ev[i + 1]));
        float ms = 0.f;
        HIPCHK(hipEventElapsedTime(&ms, m->prof_ev[i], m->prof_ev[i + 1]));
        tot += ms;
    }
    *n_launches = (int32_t)(m->prof_used / 2);
    *total_ms = tot;
    m->prof_used = 0;
    return EE_OK;
}

int ee_debug_lane_reductions(ee_model* m, int32_t* mismatches, void* stream) {
    if (!m || !mismatches) return EE_ERR_ARG;
    hipStream_t st = (hipStream_t)stream;
    EECHK(settle(m, st));
    int32_t* dev = (int32_t*)(m->ws + m->wsl.attn_part);  // (idle between steps)
    HIPCHK(hipMemsetAsync(dev, 0, 4, st));
    HIPCHK(launch_lane_reduction_check(dev, st));
    HIPCHK(hipMemcpyAsync(mismatches, dev, 4, hipMemcpyDeviceToHost, st));
    HIPCHK(hipStreamSynchronize(st));
    return EE_OK;
}

int ee_measure_stream_read(ee_model* m, size_t bytes, int n_launches, float* gb_per_s, void* stream) {
    if (!m || !gb_per_s || n_launches < 1 || n_launches > 1000) return EE_ERR_ARG;
    if (bytes == 0 || bytes > m->wl.total) bytes = m->wl.total;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0, e1;
    HIPCHK(hipEventCreate(&e0));
    hipError_t e = hipEventCreate(&e1);
    if (e == hipSuccess) e = launch_stream_read(m->wbase, bytes, nullptr, st);  // untimed first pass
    if (e == hipSuccess) e = hipEventRecord(e0, st);
    for (int i = 0; i < n_launches && e == hipSuccess; ++i) {
        // successive launches start at different offsets so a short read is not served from the caches
        const size_t off = bytes < m->wl.total ? ((size_t)i * bytes) % (m->wl.total - bytes + 1) & ~(size_t)1023 : 0;
        e = launch_stream_read(m->wbase + off, bytes, nullptr, st);
    }
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    HIPCHK(e);
    *gb_per_s = ms > 0.f ? (float)((double)(bytes / 1024 * 1024) * n_launches / (ms * 1e6)) : 0.f;
    return EE_OK;
}

int ee_model_free(ee_model* m) {
    if (!m) return EE_ERR_ARG;
    if (m->spec_ev) {
        if (m->spec_recorded) (void)hipEventSynchronize(m->spec_ev);
        (void)hipEventDestroy(m->spec_ev);
    }
    for (hipEvent_t e : m->prof_ev) (void)hipEventDestroy(e);
    if (m->pinned) (void)hipHostFree(m->pinned);
    delete m;
    return EE_OK;
}

int ee_debug_plan(int n_segments, int32_t* filled, int position, int max_pending, int refeed, int reached, int32_t* forced,
                  int32_t* row_lo, int32_t* row_hi) {
    if (n_segments < 1 || n_segments > EE_MAX_EXITS + 1 || !filled || reached >= n_segments) return EE_ERR_ARG;
    for (int k = 0; k < n_segments; ++k)
        if (filled[k] < 0 || (k && filled[k] > filled[k - 1])) return EE_ERR_STATE;
    if (forced) *forced = plan::forced(filled, n_segments, max_pending) ? 1 : 0;
    for (int k = 0; k < n_segments && row_lo && row_hi; ++k) plan::rows(filled, n_segments, k, position, refeed != 0, row_lo + k, row_hi + k);
    if (reached >= 0) {
        if (position < 0 && reached != n_segments - 1) return EE_ERR_ARG;
        if (position >= 0) plan::commit(filled, reached, position);
        else plan::flushed(filled, n_segments);
    }
    return EE_OK;
}

int ee_debug_step_confidences(const ee_model* m, int n_seqs, float* conf) {
    if (!m || !conf || n_seqs < 1 || n_seqs > EE_MAX_SEQS) return EE_ERR_ARG;
    const int n_seg = m->n_seg();
    for (int b = 0; b < n_seqs; ++b)
        for (int s = 0; s < n_seg; ++s) {
            const HeadResult& r = m->results[s * EE_MAX_SEQS + b];
            const bool fresh = m->head_tag >= m->step_tag0 ? (r.pad > m->step_tag0 && r.pad <= m->head_tag) : false;
            conf[(size_t)b * n_seg + s] = fresh ? r.conf : -1.f;
        }
    return EE_OK;
}

int ee_debug_set_logits(ee_model* m, void* dev_logits, int capacity_rows) {
    if (!m) return EE_ERR_ARG;
    m->dbg_logits = (float*)dev_logits;
    m->dbg_rows = dev_logits ? capacity_rows : 0;
    return EE_OK;
}

/* ------------------------------------------------------------------ KV cache */

int ee_kv_cache_bytes(const ee_model* m, int max_seqs, int64_t max_tokens_total, int block_tokens, int max_pending,
                      size_t* bytes) {
    EECHK(check_cache_args(m, max_seqs, max_tokens_total, block_tokens, max_pending));
    if (bytes) *bytes = kv_pool_layout(m, max_seqs, max_tokens_total, block_tokens, max_pending, 0, 0, 0, 0, 0);
    return EE_OK;
}

int ee_kv_cache_create(const ee_model* m, int max_seqs, int64_t max_tokens_total, int block_tokens, int max_pending,
                       void* dev_pool, size_t pool_bytes, ee_kv_cache** out) {
    EECHK(check_cache_args(m, max_seqs, max_tokens_total, block_tokens, max_pending));
    if (!dev_pool || !out || ((uintptr_t)dev_pool & 255)) return EE_ERR_ARG;
    ee_kv_cache* c = new (std::nothrow) ee_kv_cache();
    if (!c) return EE_ERR_NOMEM;
    size_t need = kv_pool_layout(m, max_seqs, max_tokens_total, block_tokens, max_pending, &c->n_blocks, &c->off_x, &c->off_xg,
                                 &c->off_xgh, &c->off_ssq);
    if (pool_bytes < need) {
        delete c;
        return EE_ERR_NOMEM;
    }
    const ee_config& cf = m->cfg;
    c->m = m;
    c->max_seqs = max_seqs;
    c->BT = block_tokens;
    c->S = slots_per_seq(m, max_pending);
    c->max_pending = max_pending > 0 ? max_pending : 0;
    c->pool = (char*)dev_pool;
    c->ssq_stride = cf.d_model / (16 * gemm_resid_tiles_per_wg());
    c->xs_lo = cf.dtype == EE_BF16 ? store_slots(m, max_seqs, max_pending) * cf.d_model : 0;
    c->geom.pool = dev_pool;
    c->geom.blk_stride = 2 * (size_t)cf.n_heads * block_tokens * cf.head_dim;
    c->geom.layer_stride = (size_t)c->n_blocks * c->geom.blk_stride;
    c->geom.H = cf.n_heads;
    c->geom.hd = cf.head_dim;
    c->geom.BT = block_tokens;
    c->geom.max_blocks_per_seq = m->wsl.max_blocks_per_seq;
    for (int b = c->n_blocks - 1; b >= 0; --b) c->free_blocks.push_back(b);
    c->seqs.resize(max_seqs);
    for (auto& s : c->seqs) {
        s.filled.assign(m->n_seg(), 0);
        s.tokring.assign(c->S, -1);
    }
    *out = c;
    return EE_OK;
}

int ee_kv_cache_set_refeed(ee_kv_cache* c, int on) {
    if (!c) return EE_ERR_ARG;
    const int want = on ? 1 : 0;
    if (want == c->refeed) return EE_OK;
    if (want && c->pipe.on) return EE_ERR_CONFIG;  // the fill stream resumes tokens from their saved rows
    // While a token is deferred its saved residual row means different things in the two modes (re-feeding rewrites
    // the row at whatever depth the step reached, resuming relies on it standing at the depth the watermarks say):
    // the mode may only change while no list holds a token.
    for (const SeqState& s : c->seqs)
        if (c->n_pending(s) > 0) return EE_ERR_STATE;
    c->refeed = want;
    return EE_OK;
}

int ee_kv_cache_reset(ee_kv_cache* c, int seq) {
    if (!c) return EE_ERR_ARG;
    if (seq < 0 || seq >= c->max_seqs) return EE_ERR_RANGE;
    EECHK(pipeline_drain(c));  // a fill in flight may still write to the blocks given back here
    SeqState& s = c->seqs[seq];
    for (int32_t b : s.blocks) c->free_blocks.push_back(b);
    s.blocks.clear();
    std::fill(s.filled.begin(), s.filled.end(), 0);
    std::fill(s.tokring.begin(), s.tokring.end(), -1);
    return EE_OK;
}

int ee_kv_cache_filled(const ee_kv_cache* c, int seq, int layer, int32_t* n_positions) {
    if (!c || !n_positions) return EE_ERR_ARG;
    if (seq < 0 || seq >= c->max_seqs || layer < 0 || layer >= c->m->n_kv_layers()) return EE_ERR_RANGE;
    // (the layer inside exit i is filled together with the segment that ends at that exit)
    const int L = c->m->cfg.n_layers;
    *n_positions = c->seqs[seq].filled[layer < L ? c->m->seg_of_layer(layer) : layer - L];
    return EE_OK;
}

int ee_kv_cache_pending(const ee_kv_cache* c, int seq, int32_t* n_pending) {
    if (!c || !n_pending) return EE_ERR_ARG;
    if (seq < 0 || seq >= c->max_seqs) return EE_ERR_RANGE;
    *n_pending = c->n_pending(c->seqs[seq]);
    return EE_OK;
}

int ee_kv_cache_read(ee_model* m, const ee_kv_cache* c, int seq, int layer, int pos0, int n, float* k_host, float* v_host,
                     void* stream) {
    if (!m || !c || !k_host || !v_host || c->m != m) return EE_ERR_ARG;
    if (seq < 0 || seq >= c->max_seqs || layer < 0 || layer >= m->n_kv_layers() || pos0 < 0 || n < 0) return EE_ERR_RANGE;
    const SeqState& s = c->seqs[seq];
    if (pos0 + n > (int)s.blocks.size() * c->BT) return EE_ERR_RANGE;
    if (n == 0) return EE_OK;
    EECHK(pipeline_drain(const_cast<ee_kv_cache*>(c)));
    hipStream_t st = (hipStream_t)stream;
    EECHK(settle(m, st));
    put_btab(m, c, 0, s);
    EECHK(upload(m, st));
    const size_t d = m->cfg.d_model;
    float* ks = (float*)(m->ws + m->wsl.stage);
    float* vs = ks + (size_t)m->max_rows * d;
    for (int o = 0; o < n; o += m->max_rows) {
        int nn = std::min(m->max_rows, n - o);
        HIPCHK(launch_kv_gather(m->cfg.dtype, c->geom, layer, m->dev_btab(), pos0 + o, nn, ks, vs, st));
        HIPCHK(hipMemcpyAsync(k_host + (size_t)o * d, ks, nn * d * 4, hipMemcpyDeviceToHost, st));
        HIPCHK(hipMemcpyAsync(v_host + (size_t)o * d, vs, nn * d * 4, hipMemcpyDeviceToHost, st));
        HIPCHK(hipStreamSynchronize(st));
    }
    return EE_OK;
}

int ee_debug_read_hidden(ee_model* m, const ee_kv_cache* c, int seq, float* x_host, void* stream) {
    if (!m || !c || !x_host) return EE_ERR_ARG;
    if (seq < 0 || seq >= c->max_seqs) return EE_ERR_RANGE;
    const SeqState& s = c->seqs[seq];
    if (s.filled[0] < 1) return EE_ERR_STATE;
    EECHK(pipeline_drain(const_cast<ee_kv_cache*>(c)));
    hipStream_t st = (hipStream_t)stream;
    EECHK(settle(m, st));
    size_t d = m->cfg.d_model;
    HIPCHK(hipMemcpyAsync(x_host, c->x() + (size_t)c->slot_of(seq, s.filled[0] - 1) * d, d * 4, hipMemcpyDeviceToHost, st));
    HIPCHK(hipStreamSynchronize(st));
    return EE_OK;
}

int ee_kv_cache_flush(ee_model* m, ee_kv_cache* c, int n_seqs, const int32_t* seq_ids, void* stream) {
    if (!m || !c || !seq_ids || c->m != m) return EE_ERR_ARG;
    if (n_seqs < 1 || n_seqs > m->max_seqs) return EE_ERR_ARG;
    if (m->n_missing) return EE_ERR_STATE;
    std::vector<StepSeq> ss;
    for (int b = 0; b < n_seqs; ++b) {
        int sid = seq_ids[b];
        if (sid < 0 || sid >= c->max_seqs) return EE_ERR_RANGE;
        for (auto& q : ss)
            if (q.seq == sid) return EE_ERR_ARG;
        if (c->seqs[sid].filled[0] < 1) return EE_ERR_STATE;
        ss.push_back(StepSeq{sid, -1, true, true});
    }
    if (c->pipe.on) return pipeline_drain(c);  // nothing is ever deferred there: wait for the fills in flight
    return run_step(m, c, ss, 1.0f, false, nullptr, nullptr, nullptr, (hipStream_t)stream);
}

int ee_kv_cache_free(ee_kv_cache* c) {
    if (!c) return EE_ERR_ARG;
    // (kernels that a step enqueued ahead of an exit decision may still write K and V; the model, and with it their
    // event, may already be gone)
    if (c->spec_used) (void)hipDeviceSynchronize();
    if (c->pipe.events_made) {
        if (c->pipe.on) (void)hipStreamSynchronize(c->pipe.stream);
        for (auto& e : c->pipe.slot_done) (void)hipEventDestroy(e);
        for (auto& e : c->pipe.pool) (void)hipEventDestroy(e);
        (void)hipHostFree(c->pipe.pinned);
    }
    delete c;
    return EE_OK;
}

/* ------------------------------------------------------------------ prefill */

namespace {
int prefill_impl(ee_model* m, ee_kv_cache* c, int seq, const int32_t* tokens, int n_tokens, float threshold, int32_t* next_token,
                 int32_t* exit_layer, float* conf, int32_t* score_tok, float* score_conf, float* score_nll, void* stream);
}

int ee_prefill(ee_model* m, ee_kv_cache* c, int seq, const int32_t* tokens, int n_tokens, float threshold,
               int32_t* next_token, int32_t* exit_layer, float* conf, void* stream) {
    return prefill_impl(m, c, seq, tokens, n_tokens, threshold, next_token, exit_layer, conf, nullptr, nullptr, nullptr, stream);
}

int ee_prefill_scored(ee_model* m, ee_kv_cache* c, int seq, const int32_t* tokens, int n_tokens, float threshold,
                      int32_t* next_token, int32_t* exit_layer, float* conf, int32_t* pos_token, float* pos_conf, float* pos_nll,
                      void* stream) {
    if (!pos_token || !pos_conf) return EE_ERR_ARG;
    if (m && (m->wsl.pf_rows == 0 || m->exit_layer())) return EE_ERR_CONFIG;
    return prefill_impl(m, c, seq, tokens, n_tokens, threshold, next_token, exit_layer, conf, pos_token, pos_conf, pos_nll, stream);
}

namespace {
int prefill_impl(ee_model* m, ee_kv_cache* c, int seq, const int32_t* tokens, int n_tokens, float threshold, int32_t* next_token,
                 int32_t* exit_layer, float* conf, int32_t* score_tok, float* score_conf, float* score_nll, void* stream) {
    if (!m || !c || !tokens || !next_token || !exit_layer || c->m != m) return EE_ERR_ARG;
    if (m->n_missing) return EE_ERR_STATE;
    if (seq < 0 || seq >= c->max_seqs) return EE_ERR_RANGE;
    if (n_tokens < 1 || n_tokens > m->cfg.max_positions) return EE_ERR_RANGE;
    for (int i = 0; i < n_tokens; ++i)
        if (tokens[i] < 0 || tokens[i] >= m->cfg.vocab) return EE_ERR_RANGE;
    SeqState& s = c->seqs[seq];
    if (s.filled[0] != 0) return EE_ERR_STATE;
    EECHK(ensure_blocks(c, s, n_tokens));
    hipStream_t st = (hipStream_t)stream;
    EECHK(settle(m, st));
    const ee_config& cf = m->cfg;
    const int n_seg = m->n_seg();
    const int CH = std::min(m->max_rows, 64);
    const bool large = m->wsl.pf_rows > 0 && (score_tok != nullptr || n_tokens >= PF_MIN_TOKENS);
    if (large) EECHK(prefill_large(m, c, seq, tokens, n_tokens, threshold, score_tok, score_conf, score_nll, st));
    put_btab(m, c, 0, s);
    for (int p0 = 0; p0 < n_tokens && !large; p0 += CH) {
        int n = std::min(CH, n_tokens - p0);
        bool last = p0 + n == n_tokens;
        SegDesc* d = m->host_desc(0);
        d->T = n;
        d->n_qt = 0;
        for (int r = 0; r < n; ++r) {
            d->xrow[r] = c->transient_slot(r);
            d->pos[r] = p0 + r;
            d->kvblk[r] = s.blocks[(p0 + r) / c->BT];
            d->rseq[r] = 0;
            m->host_tokens()[r] = tokens[p0 + r];
        }
        for (int r = 0; r < n; r += 16) {
            d->qt_row0[d->n_qt] = r;
            d->qt_nq[d->n_qt] = std::min(16, n - r);
            d->qt_pos0[d->n_qt] = p0 + r;
            d->qt_seq[d->n_qt] = 0;
            for (int q = 0; q < d->qt_nq[d->n_qt]; ++q) d->row_qt[r + q] = d->n_qt * 16 + q;
            ++d->n_qt;
        }
        if (last) d->xrow[n - 1] = c->slot_of(seq, n_tokens - 1);  // so that the newest hidden state can be read back
        d->n_head = 1;
        d->head_xrow[0] = d->xrow[n - 1];
        d->head_slot[0] = 0;
        // one descriptor per head so that each writes its own result slot
        for (int i = 1; i < n_seg; ++i) {
            SegDesc* di = m->host_desc(i);
            di->T = 0;
            di->n_head = 1;
            di->head_xrow[0] = d->head_xrow[0];
            di->head_slot[0] = i * EE_MAX_SEQS;
        }
        for (int i = 0; i < n_seg; ++i) fill_mlp_desc(m, c, i);
        for (int i = 0; m->exit_layer() && i < cf.n_exits; ++i) {  // each exit's layer works on copies of the chunk's rows
            fill_exit_layer_desc(m, c, i, d);
            SegDesc* e = m->host_desc(m->mlp_desc(i));
            e->n_head = 1;
            e->head_xrow[0] = c->exit_slot(n - 1);
            e->head_slot[0] = i * EE_MAX_SEQS;
        }
        EECHK(upload(m, st));
        HIPCHK(launch_embed(cf.dtype, m->wbase + m->wl.embed, m->dev_tokens(), m->dev_desc(0), n, cf.d_model, m->gain(m->wl.g1[0]),
                            c->x(), c->xg(), c->xs_lo, c->ssq(), c->ssq_stride, st));
        for (int sgi = 0; sgi < n_seg; ++sgi) {
            EECHK(run_layers(m, c, 0, n, d->n_qt, m->seg_begin(sgi), m->seg_end(sgi), p0 + n, st));
            bool fin = sgi == n_seg - 1;
            if (!fin && m->exit_layer())
                EECHK(run_exit_layer(m, c, sgi, (const int32_t*)((char*)m->dev_desc(0) + offsetof(SegDesc, xrow)),
                                     last && threshold < 1.0f, p0 + n, st));
            if (last && (fin || threshold < 1.0f)) EECHK(run_head(m, c, sgi, sgi, 1, fin ? HEAD_EMIT : HEAD_RULE, threshold, st));
        }
        HIPCHK(hipStreamSynchronize(st));  // the pinned staging is rewritten by the next chunk
    }
    int chosen = n_seg - 1;
    for (int i = 0; i < n_seg; ++i) {
        bool fin = i == n_seg - 1;
        if (!fin && !(threshold < 1.0f)) {
            if (conf) conf[i] = -1.f;
            continue;
        }
        const HeadResult& r = m->results[i * EE_MAX_SEQS];
        if (conf) conf[i] = r.conf;
        if (!fin && r.fired && chosen == n_seg - 1) chosen = i;
    }
    *next_token = m->results[chosen * EE_MAX_SEQS].token;
    *exit_layer = m->seg_end(chosen);
    for (auto& f : s.filled) f = n_tokens;
    return EE_OK;
}
}  // namespace

/* ------------------------------------------------------------------ decode */

}  // extern "C" (the static workspace below has internal linkage)

namespace {

// Step workspace of ee_decode_step_static: one array per GPU, in that GPU's memory from the moment the library's code
// is loaded there until the process ends.  In host code `static_step_ws` only names the symbol; its device address
// is looked up once per device (static_ws_of) and every use goes through that pointer.
static __device__ __align__(256) unsigned char static_step_ws[EE_STATIC_WORKSPACE_BYTES];

constexpr int STATIC_WS_MAX_DEVICES = 64;
char* g_static_ws[STATIC_WS_MAX_DEVICES];  // device address of static_step_ws on device i, or null: not looked up yet

int static_ws_of(char** out) {
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_WS_MAX_DEVICES) return EE_ERR_ARG;
    char* p = __atomic_load_n(&g_static_ws[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        HIPCHK(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(static_step_ws)));
        if (!p || ((uintptr_t)p & 255)) return EE_ERR_HIP;
        __atomic_store_n(&g_static_ws[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return EE_OK;
}

}  // namespace

extern "C" {

int ee_decode_step_static(ee_model* m, ee_kv_cache* c, int n_seqs, const int32_t* seq_ids, const int32_t* row_offsets,
                          const int32_t* tokens, const uint8_t* pending_mask, float threshold, int32_t* next_token,
                          int32_t* exit_layer, float* conf, void* stream) {
    if (!m) return EE_ERR_ARG;
    // Everything a decode step keeps in the workspace lies in front of the prompt-phase buffers, and every byte of it
    // that a step reads has been written earlier in the same step (descriptors, block tables and token ids by the
    // upload, activations and partial results by the kernels): nothing has to be cleared between calls.
    if (m->wsl.pf_begin > (size_t)EE_STATIC_WORKSPACE_BYTES) return EE_ERR_NOMEM;
    hipPointerAttribute_t attr;
    HIPCHK(hipPointerGetAttributes(&attr, m->wbase));
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (attr.device != dev) return EE_ERR_ARG;  // the array used is the current device's: it must be the model's
    char* ws = nullptr;
    EECHK(static_ws_of(&ws));
    char* const own = m->ws;
    m->ws = ws;
    const int rc = ee_decode_step(m, c, n_seqs, seq_ids, row_offsets, tokens, pending_mask, threshold, next_token, exit_layer,
                                  conf, stream);
    m->ws = own;
    return rc;
}

int ee_decode_step(ee_model* m, ee_kv_cache* c, int n_seqs, const int32_t* seq_ids, const int32_t* row_offsets,
                   const int32_t* tokens, const uint8_t* pending_mask, float threshold, int32_t* next_token,
                   int32_t* exit_layer, float* conf, void* stream) {
    if (!m || !c || !seq_ids || !row_offsets || !tokens || !pending_mask || !next_token || !exit_layer || c->m != m)
        return EE_ERR_ARG;
    if (n_seqs < 1 || n_seqs > m->max_seqs) return EE_ERR_ARG;
    if (m->n_missing) return EE_ERR_STATE;
    if (!(threshold >= 0.f)) return EE_ERR_ARG;
    std::vector<StepSeq> ss;
    size_t blocks_needed = 0;
    // pass 1: validate everything before touching any state
    // (the deepest segment of the step carries every row the caller lists: they must fit one launch)
    if (row_offsets[0] != 0 || row_offsets[n_seqs] > m->max_rows) return row_offsets[0] != 0 ? EE_ERR_ARG : EE_ERR_NOMEM;
    for (int b = 0; b < n_seqs; ++b) {
        int sid = seq_ids[b];
        if (sid < 0 || sid >= c->max_seqs) return EE_ERR_RANGE;
        for (auto& q : ss)
            if (q.seq == sid) return EE_ERR_ARG;
        const SeqState& s = c->seqs[sid];
        if (s.filled[0] < 1) return EE_ERR_STATE;  // not prefilled
        int r0 = row_offsets[b], r1 = row_offsets[b + 1];
        int pend = c->n_pending(s);
        if (r1 - r0 != pend + 1) return EE_ERR_STATE;
        for (int i = 0; i < pend; ++i) {
            if (pending_mask[r0 + i] != 1) return EE_ERR_STATE;
            if (tokens[r0 + i] != s.tokring[(s.filled.back() + i) % c->S]) return EE_ERR_STATE;
        }
        if (pending_mask[r1 - 1] != 0) return EE_ERR_STATE;
        int tok = tokens[r1 - 1];
        if (tok < 0 || tok >= m->cfg.vocab) return EE_ERR_RANGE;
        int p = s.filled[0];
        if (p >= m->cfg.max_positions) return EE_ERR_RANGE;
        if ((p + c->BT) / c->BT > c->geom.max_blocks_per_seq) return EE_ERR_RANGE;
        if ((p + c->BT) / c->BT > (int)s.blocks.size()) ++blocks_needed;
        if (blocks_needed > c->free_blocks.size()) return EE_ERR_NOMEM;
        ss.push_back(StepSeq{sid, p, plan::forced(s.filled.data(), (int)s.filled.size(), c->max_pending), true});
    }
    // pass 2: commit the current tokens
    for (int b = 0; b < n_seqs; ++b) {
        SeqState& s = c->seqs[ss[b].seq];
        EECHK(ensure_blocks(c, s, ss[b].p + 1));
        int tok = tokens[row_offsets[b + 1] - 1];
        s.tokring[ss[b].p % c->S] = tok;
    }
    EECHK(run_step(m, c, ss, threshold, true, next_token, exit_layer, conf, (hipStream_t)stream));
    return c->pipe.on ? pipeline_fill(m, c, ss) : EE_OK;
}

int ee_kv_cache_set_pipeline(ee_model* m, ee_kv_cache* c, void* dev_workspace, size_t workspace_bytes, void* fill_stream) {
    if (!m || !c || c->m != m) return EE_ERR_ARG;
    Pipeline& pp = c->pipe;
    EECHK(pipeline_drain(c));
    if (!dev_workspace) {  // back to KV recomputation (nothing is deferred in pipeline mode, so any time is fine)
        pp.on = false;
        return EE_OK;
    }
    if (((uintptr_t)dev_workspace & 255) || !fill_stream) return EE_ERR_ARG;
    if (workspace_bytes < m->wsl.pf_begin) return EE_ERR_NOMEM;
    if (c->refeed || c->S < Pipeline::RING + 2) return EE_ERR_CONFIG;  // a token's residual row must outlive its fill
    for (const SeqState& s : c->seqs)
        if (c->n_pending(s) > 0) return EE_ERR_STATE;
    if (!pp.events_made) {
        for (auto& e : pp.slot_done) HIPCHK(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        for (auto& e : pp.pool) HIPCHK(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        pp.slot_bytes = align_up(m->wsl.upload_bytes);
        HIPCHK(hipHostMalloc((void**)&pp.pinned, pp.slot_bytes * Pipeline::RING, hipHostMallocMapped));
        std::memset(pp.pinned, 0, pp.slot_bytes * Pipeline::RING);
        HIPCHK(hipHostGetDevicePointer((void**)&pp.pinned_dev, pp.pinned, 0));
        pp.events_made = true;
    }
    pp.stream = (hipStream_t)fill_stream;
    pp.ws = (char*)dev_workspace;
    pp.next_slot = 0;
    for (bool& u : pp.slot_used) u = false;
    for (int k = 0; k <= EE_MAX_EXITS; ++k) {
        pp.last_ev[k] = -1;
        pp.last_stream[k] = nullptr;
    }
    pp.on = true;
    return EE_OK;
}

}  // extern "C"
