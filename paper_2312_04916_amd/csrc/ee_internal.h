// Internal declarations shared by the host logic (ee_api.cpp) and the kernels (ee_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ee.h"

namespace ee {

// Per-launch row description, built on the host, copied to the device once per step.
struct SegDesc {
    int32_t T;       // rows in this launch
    int32_t n_qt;    // attention query tiles
    int32_t n_head;  // rows the head is evaluated on
    int32_t pad;
    int32_t xrow[EE_MAX_ROWS];   // residual-store slot of row r
    int32_t pos[EE_MAX_ROWS];    // position of row r in its sequence
    int32_t kvblk[EE_MAX_ROWS];  // physical KV block that holds pos[r]
    int32_t rseq[EE_MAX_ROWS];   // index of the row's sequence in this step's block-table array
    int32_t row_qt[EE_MAX_ROWS]; // 16 * (query tile of row r) + (index of row r inside that tile)
    int32_t qt_row0[EE_MAX_ROWS];  // query tile: first row, number of rows (<= 16, one sequence,
    int32_t qt_nq[EE_MAX_ROWS];    //   consecutive positions),
    int32_t qt_pos0[EE_MAX_ROWS];  //   position of its first row,
    int32_t qt_seq[EE_MAX_ROWS];   //   index of its sequence in this step's block-table array
    int32_t head_xrow[EE_MAX_SEQS];  // residual-store slot of each head row
    int32_t head_slot[EE_MAX_SEQS];  // result slot of each head row
};

// What a head evaluation reports per row (lives in pinned host memory, written by the kernel).
struct HeadResult {
    int32_t token;
    float conf;
    int32_t fired;
    int32_t pad;  // tag of the evaluation that wrote this entry, stored last (the host may poll it)
};

struct HeadPartial {
    float max, sum;
    int32_t idx, pad;
};

// Geometry of the paged cache as the kernels see it.
struct KvGeom {
    void* pool;           // [L][n_blocks]{ K: [H][BT][hd], V transposed in groups of 32 positions: [H][BT/32][hd][32] }
    size_t layer_stride;  // elements
    size_t blk_stride;    // elements: 2*H*BT*hd
    int32_t H, hd, BT, max_blocks_per_seq;
};

enum HeadMode { HEAD_RULE = 0, HEAD_EMIT = 1 };

// The next kernel launched by this thread reports its execution time through the event pair.
void set_launch_events(hipEvent_t start, hipEvent_t stop);

// ---- launch wrappers (ee_kernels.hip).  dtype: EE_F32 | EE_BF16.  All return the launch status.

hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t s);
hipError_t launch_lane_reduction_check(int32_t* dev_mismatches, hipStream_t s);
hipError_t launch_fill_f32(float* p, float v, size_t n, hipStream_t s);
hipError_t launch_copy_slots(int dtype, const int32_t* dev_src, const int32_t* dev_dst, int n, int d, float* x, void* xgh, size_t lo,
                             float* ssq, int ssq_stride, hipStream_t s);

hipError_t launch_rope_table(float* cs, int max_pos, int hd, float base, hipStream_t s);

// Repacks one matrix into the tile layout of the GEMM kernels; `mode` places the rows (see ee_kernels.hip).
enum PackMode { PACK_PLAIN = 0, PACK_ROTARY = 1, PACK_GATE = 2, PACK_UP = 3 };
hipError_t launch_pack(int dtype, const void* src, void* dst, int n_rows, int K, int mode, int hd, hipStream_t s);

// The start of a decode step in one launch: up to three ranges (16-byte units from the start of the upload region) copied
// from the host-mapped staging area to the workspace, and T rows looked up in the embedding (T = 0: the copy alone).
// tok_host / slot_host: the rows' token ids and residual-store slots for the by-value path (T <= 16);
// tok_mapped / slot_mapped: device views of the same arrays in the staging area.
hipError_t launch_step_begin(int dtype, const void* staging_mapped, void* ws_region, const uint32_t off16[3], const uint32_t n16[3],
                             int T, const int32_t* tok_host, const int32_t* slot_host, const int32_t* tok_mapped,
                             const int32_t* slot_mapped, const void* embed, int d, const float* g_next, float* x, void* xg, size_t xg_lo,
                             float* ssq, int ssq_stride, hipStream_t s);
hipError_t launch_embed(int dtype, const void* embed, const int32_t* dev_tokens, const SegDesc* desc, int T, int d,
                        const float* g_next, float* x, void* xg, size_t xg_lo, float* ssq, int ssq_stride, hipStream_t s);

struct GemmCommon {
    int dtype;
    const void* W;     // packed weights of this matrix
    int N, K;          // output features (packed rows), reduction length
    const void* A;     // activations, [rows][lda]
    size_t a_lo;       // element offset from the hi term of A to its lo term (bf16 model), else 0
    int lda;
    const int32_t* arow;  // row indirection into A (and into ssq), or NULL
    int a_packed;         // A holds dense rows in MFMA operand order [row/16][K/32][64 lanes][8] (bf16 model); arow then
                          // only indexes ssq
    const float* ssq;     // partial sums of squares [slot][ssq_stride], or NULL (no RMS scale)
    int ssq_stride, ssq_n;
    float inv_d, eps;
    int T;  // rows
    int min_wgs;  // workgroups a launch keeps when it gives a workgroup several column tiles (0: 512)
    const SegDesc* desc;
    const SegDesc* desc_host;  // host copy of *desc, or NULL: launches of up to 16 rows then carry the row indices by value
    // O projection only: A still lies as the attention kernel's split partials (att_ns splits), to be merged
    // while the rows are staged; NULL otherwise
    const float* att_part;
    int att_ns, att_H, att_hd;
};

hipError_t launch_gemm_qkv(const GemmCommon& c, void* q, size_t q_lo, const float* rope_cs, const KvGeom& kv, int layer,
                           hipStream_t s);
// xg_pk (optional, bf16 model): a second copy of the x.g operand, dense rows of this launch in packed order
hipError_t launch_gemm_resid(const GemmCommon& c, float* x, void* xg, void* xgh, size_t xs_lo, float* ssq_out,
                             const float* g_next, const float* g_head, int d, void* xg_pk, size_t xg_pk_lo, hipStream_t s);
hipError_t launch_gemm_swiglu(const GemmCommon& c, void* act, size_t act_lo, int F, bool act_packed, hipStream_t s);
// rows of a row-major two-term array (through an index list, or dense when NULL) -> packed array
hipError_t launch_pack_rows(const void* src, size_t src_lo, int ld, const int32_t* rows, int T, int K, void* dst, size_t dst_lo,
                            hipStream_t s);
hipError_t launch_gemm_head(const GemmCommon& c, HeadPartial* partials, int32_t* counter, float* logits, int mode,
                            float threshold, HeadResult* results, int tag, hipStream_t s);

hipError_t launch_attention(int dtype, const void* q, void* out, size_t io_lo, const SegDesc* desc, const SegDesc* desc_host, int T, int n_qt,
                            const int32_t* btab,
                            const KvGeom& kv, int layer, int d, float* part, int32_t* counters, int max_ctx, int* defer_ns,
                            bool out_packed, hipStream_t s);
// defer_ns != NULL: when the KV range was split, leave the partials unmerged and report the number of splits
// (the O projection then merges them, see GemmCommon::att_part); 0 is reported when `out` is complete.
bool gemm_rows_fit_lds(int dtype, int T, int K);  // true when the GEMMs stage this many rows in LDS

hipError_t launch_kv_gather(int dtype, const KvGeom& kv, int layer, const int32_t* btab_seq, int pos0, int n,
                            float* k_out, float* v_out, hipStream_t s);

// ---- prompt phase (ee_prefill.hip): many rows at once, activations in the packed operand layout
// [row/16][K/32][64 lanes][8 bf16] (hi and lo arrays), bf16 model only.
struct PfGemm {
    const void* W;    // packed weights
    int N, K;         // output features, reduction length (multiple of 32)
    const void* A_hi; // packed activations, rows padded to a multiple of 16
    const void* A_lo;
    const float* ssq; // [rows][ssq_n] partial sums of squares of the rows (RMS scale), or NULL
    int ssq_n;
    float inv_d, eps;
    int M;            // rows
};
hipError_t launch_pf_embed(const void* embed, const int32_t* dev_tokens, int M, int d, const float* g_next, float* x, void* xg_hi,
                           void* xg_lo, float* ssq, int ssq_n, hipStream_t s);
hipError_t launch_pf_qkv(const PfGemm& g, void* q_hi, void* q_lo, const float* rope_cs, const KvGeom& kv, int layer, const int32_t* bt,
                         int p0, hipStream_t s);
hipError_t launch_pf_attention(const void* q_hi, const void* q_lo, void* out_hi, void* out_lo, const KvGeom& kv, int layer,
                               const int32_t* bt, int p0, int M, int d, hipStream_t s);
hipError_t launch_pf_resid(const PfGemm& g, float* x, void* xg_hi, void* xg_lo, void* xgh_hi, void* xgh_lo, const float* g_next,
                           const float* g_head, float* ssq_out, int ssq_n_out, hipStream_t s);
hipError_t launch_pf_swiglu(const PfGemm& g, void* act_hi, void* act_lo, int F, hipStream_t s);
// head on every row: (arg max, confidence) per row into tok / conf
// ... and, if nll != NULL, nll[row] = log sum exp(z) - z[target[row]] (0 where target[row] < 0)
hipError_t launch_pf_head(const PfGemm& g, HeadPartial* partials, int32_t* tok, float* conf, const int32_t* target,
                          float* target_logit, float* nll, bool two_terms, hipStream_t s);
// one fp32 row of the residual stream -> decode-side residual store entry (row-major two-term operands)
hipError_t launch_pf_export_row(const float* x_row, int d, const float* g_a, const float* g_b, float* dx, void* dxg, void* dxgh,
                                size_t lo_off, float* dssq, int ssq_stride, hipStream_t s);

int gemm_resid_tiles_per_wg();  // G of the residual epilogue: ssq partials per row = d / (16*G)
size_t attention_part_floats(int max_rows, int H, int hd);  // scratch the attention kernel needs

}  // namespace ee
