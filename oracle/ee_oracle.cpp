// CPU oracle for early-exit decoding with KV recomputation.
//
// TEST INFRASTRUCTURE ONLY -- see ee_oracle.h.  Plain, slow, single-threaded by default (matvec rows
// may be spread over OpenMP threads; the sum inside a row never changes, so results are identical).
// Shares nothing with the HIP library.
//
// Model (decoder-only transformer, pre-RMSNorm, RoPE, SwiGLU, no biases; the paper only says "GPT
// Transformer", Section 2 / Appendix E -- the concrete block is the one the synthetic workloads fix):
//   x <- E[tok]
//   for l = 1..L:  h = rmsnorm(x; g1_l);  q,k,v = Wq h, Wk h, Wv h;  RoPE(q,k; pos) per head
//                  a = softmax_{j<=pos}(q.k_j / sqrt(hd)) v_j  per head;   x <- x + Wo a
//                  h = rmsnorm(x; g2_l);  x <- x + Wd (silu(Wg h) * (Wu h))
//   exit i (after layer e_i):  z = We_i rmsnorm(x; ge_i);  conf = max softmax(z)   (Sections 2, 5.2)
//   an exit may first pass x through modules of its own (Section 2): an MLP block, or a complete Transformer layer
//   (same block as above with the exit's weights; its attention runs over the K and V that the same exit layer
//   produced at the earlier positions); the backbone's x is not changed
//   rmsnorm(x; g) = g * x / sqrt(mean(x^2) + eps)
#include "ee_oracle.h"

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

int g_threads = 1;

inline float bf16_round(float v) {
    uint32_t u;
    std::memcpy(&u, &v, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return v;  // inf / nan unchanged
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;  // round to nearest, ties to even
    u &= 0xffff0000u;
    float r;
    std::memcpy(&r, &u, 4);
    return r;
}
inline float bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float r;
    std::memcpy(&r, &u, 4);
    return r;
}
inline float rnd(int dtype, float v) { return dtype == EO_BF16 ? bf16_round(v) : v; }

inline float wload(const float* w, size_t i) { return w[i]; }
inline float wload(const uint16_t* w, size_t i) { return bf16_to_f32(w[i]); }

// dot product: one running fp64 sum, terms added in index order
template <typename T>
double dotd(const T* w, const float* h, int K) {
    double s = 0;
    for (int k = 0; k < K; ++k) s += (double)wload(w, k) * (double)h[k];
    return s;
}

// y = W h, each output one dot product rounded once to fp32
template <typename T>
void matvec_t(const T* W, int N, int K, const float* h, float* y) {
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(g_threads) if (g_threads > 1 && (size_t)N * K > 262144)
#endif
    for (int n = 0; n < N; ++n) y[n] = (float)dotd(W + (size_t)n * K, h, K);
}

void matvec(int dtype, const void* W, int N, int K, const float* h, float* y) {
    if (dtype == EO_BF16)
        matvec_t((const uint16_t*)W, N, K, h, y);
    else
        matvec_t((const float*)W, N, K, h, y);
}

// rmsnorm(x; g)[k] = g[k] * x[k] / sqrt(mean(x^2) + eps), formed in fp64 and rounded once to fp32
void rmsnorm(const float* x, const float* g, int K, float eps, float* h) {
    double ss = 0;
    for (int k = 0; k < K; ++k) ss += (double)x[k] * (double)x[k];
    const double root = std::sqrt(ss / K + (double)eps);
    for (int k = 0; k < K; ++k) h[k] = (float)((double)g[k] * (double)x[k] / root);
}

// RoPE, half-split pairing: (i, i+hd/2), angle pos * base^(-2i/hd), positions from 0.
void rope(float* vec, int H, int hd, int pos, float base) {
    int half = hd / 2;
    for (int h = 0; h < H; ++h) {
        float* p = vec + (size_t)h * hd;
        for (int i = 0; i < half; ++i) {
            double ang = (double)pos * std::pow((double)base, -2.0 * i / hd);
            double c = std::cos(ang), s = std::sin(ang);
            double a = p[i], b = p[i + half];
            p[i] = (float)(a * c - b * s);
            p[i + half] = (float)(b * c + a * s);
        }
    }
}

void attention_row(const float* q, const float* K, const float* V, int n_ctx, int H, int hd,
                   float* out) {
    int d = H * hd;
    double scale = 1.0 / std::sqrt((double)hd);
    std::vector<float> s(n_ctx);
    std::vector<double> p(n_ctx);
    for (int h = 0; h < H; ++h) {
        const float* qh = q + (size_t)h * hd;
        float m = -INFINITY;
        for (int j = 0; j < n_ctx; ++j) {
            s[j] = (float)(dotd(K + (size_t)j * d + (size_t)h * hd, qh, hd) * scale);
            if (s[j] > m) m = s[j];
        }
        double den = 0;
        for (int j = 0; j < n_ctx; ++j) {
            p[j] = std::exp((double)s[j] - (double)m);
            den += p[j];
        }
        for (int c = 0; c < hd; ++c) {
            double acc = 0;
            for (int j = 0; j < n_ctx; ++j) acc += p[j] * (double)V[(size_t)j * d + (size_t)h * hd + c];
            out[(size_t)h * hd + c] = (float)(acc / den);
        }
    }
}

void swiglu(const float* gate, const float* up, int n, float* out) {
    for (int i = 0; i < n; ++i) {
        double t = gate[i];
        double sl = t / (1.0 + std::exp(-t));
        out[i] = (float)(sl * (double)up[i]);
    }
}

void softmax_max(const float* z, int n, eo_diag* out) {
    int a = 0;
    for (int i = 1; i < n; ++i)
        if (z[i] > z[a]) a = i;  // strict: lowest index among equals
    int b = -1;
    for (int i = 0; i < n; ++i)
        if (i != a && (b < 0 || z[i] > z[b])) b = i;
    double den = 0;
    for (int i = 0; i < n; ++i) den += std::exp((double)z[i] - (double)z[a]);
    out->argmax = a;
    out->arg2 = b;
    out->conf = (float)(1.0 / den);
    out->top1 = z[a];
    out->top2 = b >= 0 ? z[b] : -INFINITY;
}

}  // namespace

struct eo_model {
    eo_config c;
    const void* embed = nullptr;
    std::vector<const float*> g1, g2;
    std::vector<const void*> wq, wk, wv, wo, wg, wu, wd;
    std::vector<const float*> ge;
    std::vector<const void*> we;
    std::vector<const float*> gm;           // exit MLP (alone, or second half of the exit's layer): norm gain
    std::vector<const void*> ewg, ewu, ewd; // ... gate, up, down
    std::vector<const float*> ga;           // exit layer, attention half: norm gain
    std::vector<const void*> ewq, ewk, ewv, ewo;
    const float* gf = nullptr;
    const void* wf = nullptr;
    int n_seg() const { return c.n_exits + 1; }
    bool exit_layer() const { return c.exit_flags & EO_EXIT_LAYER; }
    int n_kv_layers() const { return c.n_layers + (exit_layer() ? c.n_exits : 0); }  // exit i's layer caches as layer L+i
    int seg_end(int s) const { return s < c.n_exits ? c.exit_layers[s] : c.n_layers; }
    int seg_begin(int s) const { return s == 0 ? 0 : c.exit_layers[s - 1]; }
};

namespace {

void embed_row(const eo_model* m, int tok, float* x) {
    int d = m->c.d_model;
    if (m->c.dtype == EO_BF16) {
        const uint16_t* e = (const uint16_t*)m->embed + (size_t)tok * d;
        for (int i = 0; i < d; ++i) x[i] = bf16_to_f32(e[i]);
    } else {
        std::memcpy(x, (const float*)m->embed + (size_t)tok * d, sizeof(float) * d);
    }
}

// The weights of one Transformer block: a backbone layer, or the layer an exit may contain.
struct BlockW {
    const float *g1, *g2;
    const void *wq, *wk, *wv, *wo, *wg, *wu, *wd;
};
BlockW layer_weights(const eo_model* m, int l) {
    return BlockW{m->g1[l], m->g2[l], m->wq[l], m->wk[l], m->wv[l], m->wo[l], m->wg[l], m->wu[l], m->wd[l]};
}
BlockW exit_layer_weights(const eo_model* m, int i) {
    return BlockW{m->ga[i], m->gm[i], m->ewq[i], m->ewk[i], m->ewv[i], m->ewo[i], m->ewg[i], m->ewu[i], m->ewd[i]};
}

// K and V of one row: k, v = Wk h, Wv h with h = rmsnorm(x; g1), k rotated to the row's position, both rounded to the
// storage type of the cache.  Written to row `pos` of K, V ([>= pos+1][d]); h is returned for the caller's q.
void block_kv_row(const eo_model* m, const BlockW& w, const float* x, int pos, float* K, float* V, float* h) {
    const eo_config& c = m->c;
    int d = c.d_model, dt = c.dtype;
    float* k = K + (size_t)pos * d;
    float* v = V + (size_t)pos * d;
    rmsnorm(x, w.g1, d, c.rms_eps, h);
    matvec(dt, w.wk, d, d, h, k);
    matvec(dt, w.wv, d, d, h, v);
    rope(k, c.n_heads, c.head_dim, pos, c.rope_base);
    for (int i = 0; i < d; ++i) {  // the cache stores K and V in the model's storage type
        k[i] = rnd(dt, k[i]);
        v[i] = rnd(dt, v[i]);
    }
}

// One block on one row.  K, V: [>= pos+1][d]; row pos is written, rows 0..pos are read.
void block_row(const eo_model* m, const BlockW& w, float* x, int pos, float* K, float* V) {
    const eo_config& c = m->c;
    int d = c.d_model, F = c.d_ff, dt = c.dtype;
    std::vector<float> h(d > F ? d : F), q(d), a(d), gate(F), up(F), y(d);
    block_kv_row(m, w, x, pos, K, V, h.data());
    matvec(dt, w.wq, d, d, h.data(), q.data());
    rope(q.data(), c.n_heads, c.head_dim, pos, c.rope_base);
    attention_row(q.data(), K, V, pos + 1, c.n_heads, c.head_dim, a.data());
    matvec(dt, w.wo, d, d, a.data(), y.data());
    for (int i = 0; i < d; ++i) x[i] += y[i];
    rmsnorm(x, w.g2, d, c.rms_eps, h.data());
    matvec(dt, w.wg, F, d, h.data(), gate.data());
    matvec(dt, w.wu, F, d, h.data(), up.data());
    swiglu(gate.data(), up.data(), F, h.data());
    matvec(dt, w.wd, d, F, h.data(), y.data());
    for (int i = 0; i < d; ++i) x[i] += y[i];
}

void layer_row(const eo_model* m, int l, float* x, int pos, float* K, float* V) {
    block_row(m, layer_weights(m, l), x, pos, K, V);
}

// Head `head` on one row (Section 2, "Model architectures"): an exit is, in this order, an optional MLP block,
// an optional normalisation, and an output embedding matrix that is its own or the input embedding.  (An exit that
// contains a complete Transformer layer applies that layer first, see exit_layer_row; x is then its output.)
void head_row(const eo_model* m, int head, const float* x, float* z, eo_diag* diag) {
    const eo_config& c = m->c;
    const int d = c.d_model, F = c.d_ff, dt = c.dtype;
    bool fin = head >= c.n_exits;
    const void* W = (c.exit_flags & EO_TIE_EMBEDDINGS) ? m->embed : (fin ? m->wf : m->we[head]);
    std::vector<float> xe(x, x + d), h(d > F ? d : F);
    if (!fin && (c.exit_flags & EO_EXIT_MLP)) {
        std::vector<float> gate(F), up(F), y(d);
        rmsnorm(xe.data(), m->gm[head], d, c.rms_eps, h.data());
        matvec(dt, m->ewg[head], F, d, h.data(), gate.data());
        matvec(dt, m->ewu[head], F, d, h.data(), up.data());
        swiglu(gate.data(), up.data(), F, h.data());
        matvec(dt, m->ewd[head], d, F, h.data(), y.data());
        for (int i = 0; i < d; ++i) xe[i] += y[i];
    }
    if (!fin && (c.exit_flags & EO_EXIT_NO_NORM))
        for (int i = 0; i < d; ++i) h[i] = xe[i];
    else
        rmsnorm(xe.data(), fin ? m->gf : m->ge[head], d, c.rms_eps, h.data());
    matvec(dt, W, c.vocab, d, h.data(), z);
    if (diag) {
        softmax_max(z, c.vocab, diag);
        diag->layer = fin ? c.n_layers : c.exit_layers[head];
    }
}

}  // namespace

struct eo_state {
    const eo_model* m;
    int max_pos, max_pending;
    std::vector<int32_t> tok;
    std::vector<int> filled;
    std::vector<float> K, V;  // [L][max_pos][d]
    bool in_step = false, forced = false;
    int cur_pos = 0, seg_cursor = 0, row_pos0 = 0;
    std::vector<float> rows;  // [n_rows][d]
    std::vector<float> last_hidden, last_logits;
    float* Kl(int l) { return K.data() + (size_t)l * max_pos * m->c.d_model; }
    float* Vl(int l) { return V.data() + (size_t)l * max_pos * m->c.d_model; }
    int n_rows() const { return cur_pos - row_pos0 + 1; }
};

namespace {

// Exit `i` on the row x at position pos of the state's sequence.  If the exit contains a Transformer layer, the row's
// K and V in that layer are written (cache layer L+i) whether or not the head is read; with_head: the exit's layer
// (on a copy of x), then the head, into last_logits and *diag.
void exit_row(eo_state* s, int i, const float* x, int pos, bool with_head, eo_diag* diag) {
    const eo_model* m = s->m;
    const int d = m->c.d_model, L = m->c.n_layers;
    std::vector<float> xe(x, x + d);
    if (m->exit_layer()) {
        BlockW w = exit_layer_weights(m, i);
        if (with_head) {
            block_row(m, w, xe.data(), pos, s->Kl(L + i), s->Vl(L + i));
        } else {
            std::vector<float> h(d);
            block_kv_row(m, w, x, pos, s->Kl(L + i), s->Vl(L + i), h.data());
        }
    }
    if (with_head) head_row(m, i, xe.data(), s->last_logits.data(), diag);
}

}  // namespace

extern "C" {

int eo_exit_layer_sequence(const eo_model* m, int exit, const float* hidden, int n, float* x_out, float* k_out, float* v_out) {
    if (!m->exit_layer() || exit < 0 || exit >= m->c.n_exits || n < 1) return -1;
    const int d = m->c.d_model;
    std::vector<float> K((size_t)n * d), V((size_t)n * d);
    BlockW w = exit_layer_weights(m, exit);
    for (int t = 0; t < n; ++t) {
        std::vector<float> x(hidden + (size_t)t * d, hidden + (size_t)(t + 1) * d);
        block_row(m, w, x.data(), t, K.data(), V.data());
        if (x_out) std::memcpy(x_out + (size_t)t * d, x.data(), sizeof(float) * d);
    }
    if (k_out) std::memcpy(k_out, K.data(), sizeof(float) * n * d);
    if (v_out) std::memcpy(v_out, V.data(), sizeof(float) * n * d);
    return 0;
}

void eo_set_threads(int n) { g_threads = n < 1 ? 1 : n; }
int eo_get_threads(void) { return g_threads; }
float eo_bf16_round(float v) { return bf16_round(v); }

eo_model* eo_model_create(const eo_config* cfg) {
    const eo_config& c = *cfg;
    if (c.n_layers < 1 || c.d_model < 1 || c.n_heads < 1 || c.head_dim < 2 || (c.head_dim & 1) ||
        c.n_heads * c.head_dim != c.d_model || c.d_ff < 1 || c.vocab < 2 || c.n_exits < 0 || c.n_exits > 8 ||
        (c.exit_flags & ~(EO_EXIT_NO_NORM | EO_TIE_EMBEDDINGS | EO_EXIT_MLP | EO_EXIT_LAYER)) ||
        ((c.exit_flags & EO_EXIT_MLP) && (c.exit_flags & EO_EXIT_LAYER)))
        return nullptr;
    for (int i = 0; i < c.n_exits; ++i) {
        if (c.exit_layers[i] < 1 || c.exit_layers[i] >= c.n_layers) return nullptr;
        if (i && c.exit_layers[i] <= c.exit_layers[i - 1]) return nullptr;
    }
    eo_model* m = new eo_model;
    m->c = c;
    int L = c.n_layers;
    m->g1.assign(L, nullptr);
    m->g2.assign(L, nullptr);
    for (auto* v : {&m->wq, &m->wk, &m->wv, &m->wo, &m->wg, &m->wu, &m->wd}) v->assign(L, nullptr);
    m->ge.assign(c.n_exits, nullptr);
    m->we.assign(c.n_exits, nullptr);
    m->gm.assign(c.n_exits, nullptr);
    m->ga.assign(c.n_exits, nullptr);
    for (auto* v : {&m->ewg, &m->ewu, &m->ewd, &m->ewq, &m->ewk, &m->ewv, &m->ewo}) v->assign(c.n_exits, nullptr);
    return m;
}

int eo_model_set_tensor(eo_model* m, int kind, int index, const void* data) {
    int L = m->c.n_layers, E = m->c.n_exits;
    auto lay = [&](int n) { return index >= 0 && index < n; };
    switch (kind) {
        case EO_EMBED: m->embed = data; return 0;
        case EO_ATTN_NORM: if (!lay(L)) return -1; m->g1[index] = (const float*)data; return 0;
        case EO_MLP_NORM: if (!lay(L)) return -1; m->g2[index] = (const float*)data; return 0;
        case EO_WQ: if (!lay(L)) return -1; m->wq[index] = data; return 0;
        case EO_WK: if (!lay(L)) return -1; m->wk[index] = data; return 0;
        case EO_WV: if (!lay(L)) return -1; m->wv[index] = data; return 0;
        case EO_WO: if (!lay(L)) return -1; m->wo[index] = data; return 0;
        case EO_WG: if (!lay(L)) return -1; m->wg[index] = data; return 0;
        case EO_WU: if (!lay(L)) return -1; m->wu[index] = data; return 0;
        case EO_WD: if (!lay(L)) return -1; m->wd[index] = data; return 0;
        case EO_EXIT_NORM: if (!lay(E)) return -1; m->ge[index] = (const float*)data; return 0;
        case EO_EXIT_HEAD: if (!lay(E)) return -1; m->we[index] = data; return 0;
        case EO_FINAL_NORM: m->gf = (const float*)data; return 0;
        case EO_FINAL_HEAD: m->wf = data; return 0;
        case EO_EXIT_MLP_NORM: if (!lay(E)) return -1; m->gm[index] = (const float*)data; return 0;
        case EO_EXIT_WG: if (!lay(E)) return -1; m->ewg[index] = data; return 0;
        case EO_EXIT_WU: if (!lay(E)) return -1; m->ewu[index] = data; return 0;
        case EO_EXIT_WD: if (!lay(E)) return -1; m->ewd[index] = data; return 0;
        case EO_EXIT_ATTN_NORM: if (!lay(E)) return -1; m->ga[index] = (const float*)data; return 0;
        case EO_EXIT_WQ: if (!lay(E)) return -1; m->ewq[index] = data; return 0;
        case EO_EXIT_WK: if (!lay(E)) return -1; m->ewk[index] = data; return 0;
        case EO_EXIT_WV: if (!lay(E)) return -1; m->ewv[index] = data; return 0;
        case EO_EXIT_WO: if (!lay(E)) return -1; m->ewo[index] = data; return 0;
    }
    return -1;
}

void eo_model_free(eo_model* m) { delete m; }

/* ------------------------------------------------------------------ G0 */

int eo_forward_sequence(const eo_model* m, const int32_t* tokens, int n, float* hidden_out, float* k_out,
                        float* v_out) {
    const eo_config& c = m->c;
    int d = c.d_model, L = c.n_layers;
    std::vector<float> X((size_t)n * d), K((size_t)n * d), V((size_t)n * d);
    for (int t = 0; t < n; ++t) {
        if (tokens[t] < 0 || tokens[t] >= c.vocab) return -1;
        embed_row(m, tokens[t], X.data() + (size_t)t * d);
    }
    if (hidden_out) std::memcpy(hidden_out, X.data(), sizeof(float) * n * d);
    for (int l = 0; l < L; ++l) {  // layer-major: the whole sequence through layer l, then l+1
        for (int t = 0; t < n; ++t) layer_row(m, l, X.data() + (size_t)t * d, t, K.data(), V.data());
        if (hidden_out) std::memcpy(hidden_out + (size_t)(l + 1) * n * d, X.data(), sizeof(float) * n * d);
        if (k_out) std::memcpy(k_out + (size_t)l * n * d, K.data(), sizeof(float) * n * d);
        if (v_out) std::memcpy(v_out + (size_t)l * n * d, V.data(), sizeof(float) * n * d);
    }
    return 0;
}

// The plain definition: each new token from a cache-free forward of everything so far.  max_pending
// reproduces the forced full-depth rule from the exit history alone (a decode step is forced when the
// number of early-exited tokens since the last full-depth one has reached max_pending; <= 0: never).
static int generate_g0(const eo_model* m, const int32_t* prompt, int n_prompt, int n_new, float threshold,
                       int max_pending, int32_t* tokens_out, int32_t* exit_layer_out) {
    const eo_config& c = m->c;
    int d = c.d_model, L = c.n_layers;
    std::vector<int32_t> seq(prompt, prompt + n_prompt);
    std::vector<float> z(c.vocab);
    int pending = 0;
    for (int j = 0; j < n_new; ++j) {
        int n = (int)seq.size();
        std::vector<float> hid((size_t)(L + 1) * n * d);
        if (eo_forward_sequence(m, seq.data(), n, hid.data(), nullptr, nullptr)) return -1;
        bool forced = j > 0 && max_pending > 0 && pending >= max_pending;
        int tok = -1, ex = L;
        if (threshold < 1.0f && !forced) {
            for (int i = 0; i < c.n_exits && tok < 0; ++i) {
                const float* x = hid.data() + ((size_t)c.exit_layers[i] * n + (n - 1)) * d;
                eo_diag dg;
                std::vector<float> xe;
                if (m->exit_layer()) {  // the exit's own layer over the whole sequence of hidden states at this depth
                    xe.resize((size_t)n * d);
                    if (eo_exit_layer_sequence(m, i, hid.data() + (size_t)c.exit_layers[i] * n * d, n, xe.data(), nullptr, nullptr))
                        return -1;
                    x = xe.data() + (size_t)(n - 1) * d;
                }
                head_row(m, i, x, z.data(), &dg);
                if (dg.conf >= threshold) {
                    tok = dg.argmax;
                    ex = c.exit_layers[i];
                }
            }
        }
        if (tok < 0) {
            const float* x = hid.data() + ((size_t)L * n + (n - 1)) * d;
            eo_diag dg;
            head_row(m, c.n_exits, x, z.data(), &dg);
            tok = dg.argmax;
        }
        if (j > 0) pending = (ex == L) ? 0 : pending + 1;  // token j-1's position was processed to depth ex
        tokens_out[j] = tok;
        exit_layer_out[j] = ex;
        seq.push_back(tok);
    }
    return 0;
}

int eo_generate_g0(const eo_model* m, const int32_t* prompt, int n_prompt, int n_new, float threshold,
                   int32_t* tokens_out, int32_t* exit_layer_out) {
    return generate_g0(m, prompt, n_prompt, n_new, threshold, 0, tokens_out, exit_layer_out);
}

int eo_generate_g0_capped(const eo_model* m, const int32_t* prompt, int n_prompt, int n_new,
                          float threshold, int max_pending, int32_t* tokens_out, int32_t* exit_layer_out) {
    return generate_g0(m, prompt, n_prompt, n_new, threshold, max_pending, tokens_out, exit_layer_out);
}

// A standard LLM: incremental KV cache, no exits at all.
int eo_generate_plain(const eo_model* m, const int32_t* prompt, int n_prompt, int n_new,
                      int32_t* tokens_out) {
    const eo_config& c = m->c;
    int d = c.d_model, L = c.n_layers, maxp = n_prompt + n_new;
    std::vector<float> K((size_t)L * maxp * d), V((size_t)L * maxp * d), x(d), z(c.vocab);
    int tok = -1;
    for (int t = 0; t < n_prompt + n_new - 1; ++t) {
        int in = t < n_prompt ? prompt[t] : tokens_out[t - n_prompt];
        embed_row(m, in, x.data());
        for (int l = 0; l < L; ++l)
            layer_row(m, l, x.data(), t, K.data() + (size_t)l * maxp * d, V.data() + (size_t)l * maxp * d);
        if (t >= n_prompt - 1) {
            eo_diag dg;
            head_row(m, c.n_exits, x.data(), z.data(), &dg);
            tok = dg.argmax;
            tokens_out[t - (n_prompt - 1)] = tok;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ G1 */

eo_state* eo_state_create(const eo_model* m, int max_positions, int max_pending) {
    if (!m || max_positions < 1) return nullptr;
    eo_state* s = new eo_state;
    s->m = m;
    s->max_pos = max_positions;
    s->max_pending = max_pending;
    s->tok.assign(max_positions, -1);
    s->filled.assign(m->n_seg(), 0);
    size_t n = (size_t)m->n_kv_layers() * max_positions * m->c.d_model;
    s->K.assign(n, 0.f);
    s->V.assign(n, 0.f);
    s->last_hidden.assign(m->c.d_model, 0.f);
    s->last_logits.assign(m->c.vocab, 0.f);
    return s;
}

void eo_state_free(eo_state* s) { delete s; }

int eo_prefill(eo_state* s, const int32_t* tokens, int n, eo_diag* diag_out) {
    const eo_model* m = s->m;
    const eo_config& c = m->c;
    if (s->in_step || s->filled[0] != 0 || n < 1 || n > s->max_pos) return -1;
    int d = c.d_model;
    std::vector<float> x(d);
    for (int t = 0; t < n; ++t) {
        if (tokens[t] < 0 || tokens[t] >= c.vocab) return -1;
        s->tok[t] = tokens[t];
        embed_row(m, tokens[t], x.data());
        int next_exit = 0;
        for (int l = 0; l < c.n_layers; ++l) {
            layer_row(m, l, x.data(), t, s->Kl(l), s->Vl(l));
            if (next_exit < c.n_exits && c.exit_layers[next_exit] == l + 1) {
                // every position leaves its K and V in the exit's own layer; the head is read at the last one
                if (t == n - 1)
                    exit_row(s, next_exit, x.data(), t, true, &diag_out[next_exit]);
                else if (m->exit_layer())
                    exit_row(s, next_exit, x.data(), t, false, nullptr);
                ++next_exit;
            }
        }
        if (t == n - 1) {
            head_row(m, c.n_exits, x.data(), s->last_logits.data(), &diag_out[c.n_exits]);
            s->last_hidden = x;
        }
    }
    for (auto& f : s->filled) f = n;
    return 0;
}

int eo_step_begin(eo_state* s, int32_t token) {
    const eo_model* m = s->m;
    if (s->in_step || token < 0 || token >= m->c.vocab) return -1;
    int p = s->filled[0];
    if (p >= s->max_pos || p == 0) return -1;
    int last = m->n_seg() - 1;
    int pending = s->filled[0] - s->filled[last];
    s->forced = s->max_pending > 0 && pending >= s->max_pending;
    s->tok[p] = token;
    s->cur_pos = p;
    s->row_pos0 = s->filled[last];  // the most recent tokens with missing deep KV, then the current one
    int d = m->c.d_model;
    s->rows.assign((size_t)s->n_rows() * d, 0.f);
    for (int i = 0; i < s->n_rows(); ++i) embed_row(m, s->tok[s->row_pos0 + i], s->rows.data() + (size_t)i * d);
    s->seg_cursor = 0;
    s->in_step = true;
    return s->forced ? 1 : 0;
}

int eo_step_advance(eo_state* s, int eval_head, eo_diag* diag) {
    const eo_model* m = s->m;
    if (!s->in_step || s->seg_cursor >= m->n_seg()) return -1;
    int d = m->c.d_model, seg = s->seg_cursor;
    for (int l = m->seg_begin(seg); l < m->seg_end(seg); ++l)
        for (int i = 0; i < s->n_rows(); ++i)  // oldest first: a row attends to the rows before it
            layer_row(m, l, s->rows.data() + (size_t)i * d, s->row_pos0 + i, s->Kl(l), s->Vl(l));
    s->seg_cursor = seg + 1;
    const float* xc = s->rows.data() + (size_t)(s->n_rows() - 1) * d;
    std::memcpy(s->last_hidden.data(), xc, sizeof(float) * d);
    int depth = m->seg_end(seg);
    if (depth == m->c.n_layers) {
        head_row(m, m->c.n_exits, xc, s->last_logits.data(), diag);
    } else {
        // the deferred rows (oldest first) leave their K and V in the exit's own layer, if it has one; the current
        // row does too, and is the only one whose head is read (and only if the exits are on in this step)
        if (m->exit_layer())
            for (int i = 0; i + 1 < s->n_rows(); ++i)
                exit_row(s, seg, s->rows.data() + (size_t)i * d, s->row_pos0 + i, false, nullptr);
        if (eval_head || m->exit_layer()) exit_row(s, seg, xc, s->cur_pos, eval_head != 0, diag);
    }
    return depth;
}

int eo_step_commit(eo_state* s, int32_t token) {
    if (!s->in_step || s->seg_cursor < 1) return -1;
    (void)token;
    for (int sg = 0; sg < s->seg_cursor; ++sg) s->filled[sg] = s->cur_pos + 1;
    s->in_step = false;
    return 0;
}

int eo_decode_step(eo_state* s, int32_t token, float threshold, int32_t* next_token, int32_t* exit_layer,
                   float* conf) {
    int forced = eo_step_begin(s, token);
    if (forced < 0) return -1;
    bool eval = !forced && threshold < 1.0f;
    for (;;) {
        eo_diag dg;
        int depth = eo_step_advance(s, eval, &dg);
        if (depth < 0) return -1;
        if (depth == s->m->c.n_layers || (eval && dg.conf >= threshold)) {
            *next_token = dg.argmax;
            *exit_layer = depth;
            if (conf) *conf = dg.conf;
            return eo_step_commit(s, dg.argmax);
        }
    }
}

int eo_flush(eo_state* s) {
    const eo_model* m = s->m;
    if (s->in_step) return -1;
    int last = m->n_seg() - 1, d = m->c.d_model;
    int p0 = s->filled[last], p1 = s->filled[0];
    std::vector<float> x(d);
    for (int t = p0; t < p1; ++t) {
        embed_row(m, s->tok[t], x.data());
        int next_exit = 0;
        for (int l = 0; l < m->c.n_layers; ++l) {
            layer_row(m, l, x.data(), t, s->Kl(l), s->Vl(l));
            if (next_exit < m->c.n_exits && m->c.exit_layers[next_exit] == l + 1) {
                if (m->exit_layer()) exit_row(s, next_exit, x.data(), t, false, nullptr);
                ++next_exit;
            }
        }
    }
    for (auto& f : s->filled) f = p1;
    return 0;
}

int eo_filled(const eo_state* s, int segment) {
    if (segment < 0 || segment >= s->m->n_seg()) return -1;
    return s->filled[segment];
}

int eo_n_pending(const eo_state* s) { return s->filled[0] - s->filled[s->m->n_seg() - 1]; }

int eo_kv_read(const eo_state* s, int layer, int pos0, int n, float* k_out, float* v_out) {
    const eo_config& c = s->m->c;
    if (layer < 0 || layer >= s->m->n_kv_layers() || pos0 < 0 || n < 0 || pos0 + n > s->max_pos) return -1;
    size_t off = ((size_t)layer * s->max_pos + pos0) * c.d_model;
    std::memcpy(k_out, s->K.data() + off, sizeof(float) * n * c.d_model);
    std::memcpy(v_out, s->V.data() + off, sizeof(float) * n * c.d_model);
    return 0;
}

int eo_last_hidden(const eo_state* s, float* x_out) {
    std::memcpy(x_out, s->last_hidden.data(), sizeof(float) * s->m->c.d_model);
    return 0;
}

int eo_last_logits(const eo_state* s, float* z_out) {
    std::memcpy(z_out, s->last_logits.data(), sizeof(float) * s->m->c.vocab);
    return 0;
}

/* ------------------------------------------------------------------ single operations */

void eo_norm_matvec(int dtype, const void* W, int N, int K, const float* x, const float* g, float eps,
                    float* y) {
    std::vector<float> h(K);
    if (g)
        rmsnorm(x, g, K, eps, h.data());
    else
        for (int k = 0; k < K; ++k) h[k] = x[k];
    matvec(dtype, W, N, K, h.data(), y);
}

void eo_rope(float* vec, int n_heads, int head_dim, int pos, float base) {
    rope(vec, n_heads, head_dim, pos, base);
}

void eo_attention_row(const float* q, const float* K, const float* V, int n_ctx, int n_heads,
                      int head_dim, float* out) {
    attention_row(q, K, V, n_ctx, n_heads, head_dim, out);
}

void eo_swiglu(const float* gate, const float* up, int n, float* out) {
    swiglu(gate, up, n, out);
}

void eo_softmax_max(const float* z, int n, eo_diag* out) {
    softmax_max(z, n, out);
    out->layer = -1;
}

int eo_layer_row(const eo_model* m, int layer, float* x, int pos, float* K, float* V) {
    if (layer < 0 || layer >= m->c.n_layers || pos < 0) return -1;
    layer_row(m, layer, x, pos, K, V);
    return 0;
}

int eo_head_row(const eo_model* m, int head, const float* x, float* z_out, eo_diag* diag) {
    if (head < 0 || head > m->c.n_exits) return -1;
    std::vector<float> z;
    if (!z_out) {
        z.resize(m->c.vocab);
        z_out = z.data();
    }
    head_row(m, head, x, z_out, diag);
    return 0;
}

}  // extern "C"
