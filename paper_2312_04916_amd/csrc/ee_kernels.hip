// HIP kernels (gfx950) for one early-exit decode step with KV recomputation.
//
// Every decode GEMM has at most a few dozen rows (the current token plus the deferred tokens that are
// carried along, Section 4 "KV recomputation"), so it is a weight-streaming problem bound by HBM
// bandwidth: weights are stored pre-shuffled so that one wave load instruction fetches 1 KB of
// contiguous memory that is already a 16x32 bf16 MFMA operand, a workgroup owns a few 16-column
// tiles and splits the reduction dimension over its waves, and everything that follows the product
// (rotary embedding and the KV-cache write, residual add, the next layer's normalised input,
// SwiGLU, the soft-max max/arg-max over the vocabulary and the exit decision) runs in the epilogue
// of the kernel that produced it.  No float atomics: every reduction has a fixed order.
#include "ee_internal.h"

#include <hip/hip_ext.h>

namespace ee {

// Optional timing of the next launch: the event pair is attached to the dispatch itself, so the
// elapsed time between the two events is the kernel's own execution time.
static thread_local hipEvent_t t_ev0 = nullptr, t_ev1 = nullptr;
void set_launch_events(hipEvent_t start, hipEvent_t stop) {
    t_ev0 = start;
    t_ev1 = stop;
}
#define EE_LAUNCH(kernel, grid, block, stream, ...)                                            \
    do {                                                                                       \
        if (t_ev0) {                                                                           \
            hipEvent_t _a = t_ev0, _b = t_ev1;                                                 \
            t_ev0 = t_ev1 = nullptr;                                                           \
            hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, _a, _b, 0, __VA_ARGS__);     \
        } else {                                                                               \
            hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);                   \
        }                                                                                      \
    } while (0)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <typename ST> __device__ __forceinline__ ST cvt_st(float v);
template <> __device__ __forceinline__ float cvt_st<float>(float v) { return v; }
template <> __device__ __forceinline__ __bf16 cvt_st<__bf16>(float v) { return (__bf16)v; }  // round to nearest even

// Activations of the bf16 model are carried as two bf16 terms, hi = bf16(v) and lo = bf16(v - hi), so
// that a matrix input keeps about 16 mantissa bits while still being an MFMA bf16 operand (two MFMAs
// per tile; the matrix cores idle anyway in this bandwidth-bound regime).  `lo_off` is the element
// distance from the hi array to the lo array.  The fp32 model has a single term.
template <typename ST> __device__ __forceinline__ void store_split(ST* p, size_t lo_off, float v);
template <> __device__ __forceinline__ void store_split<float>(float* p, size_t, float v) { *p = v; }
template <> __device__ __forceinline__ void store_split<__bf16>(__bf16* p, size_t lo_off, float v) {
    __bf16 hi = (__bf16)v;
    p[0] = hi;
    p[lo_off] = (__bf16)(v - (float)hi);
}
template <typename ST> __device__ __forceinline__ float load_split(const ST* p, size_t lo_off);
template <> __device__ __forceinline__ float load_split<float>(const float* p, size_t) { return *p; }
template <> __device__ __forceinline__ float load_split<__bf16>(const __bf16* p, size_t lo_off) {
    return (float)p[0] + (float)p[lo_off];
}

// ------------------------------------------------------------------------------------------------
// rotary table: cs[pos][i] = (cos, sin)(pos * base^(-2i/hd)), evaluated in fp64
// ------------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(float2* cs, int max_pos, int half, int hd, float base) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= max_pos * half) return;
    int pos = idx / half, i = idx % half;
    double ang = (double)pos * pow((double)base, -2.0 * (double)i / (double)hd);
    cs[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

hipError_t launch_rope_table(float* cs, int max_pos, int hd, float base, hipStream_t s) {
    int n = max_pos * (hd / 2);
    EE_LAUNCH(rope_table_kernel, dim3((n + 255) / 256), dim3(256), s, (float2*)cs, max_pos, hd / 2, hd, base);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// weight packing.  Source: row-major [n_rows][K].  Destination rows are grouped in tiles of 16.
//   bf16: [tile][K/32][lane 0..63][8]  with lane = (k_group << 4) | row_in_tile, k = kt*32 + k_group*8 + j
//   fp32: [tile][16][K] (row permutation only)
// mode 1 reorders the 16-row tiles inside every head so that the two halves of a rotary pair
// (feature i and i + hd/2) sit in neighbouring tiles: tile (h, c, s) = features h*hd + s*hd/2 + c*16 ..
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int dst_tile_of(int src_tile, int mode, int hd, int tile_mul, int tile_off) {
    if (mode == 0) return src_tile * tile_mul + tile_off;
    int row = src_tile * 16;
    int h = row / hd, o = row % hd;
    int s = o >= hd / 2;
    int c = (o % (hd / 2)) / 16;
    return (h * (hd / 32) + c) * 2 + s;
}

__global__ void pack_bf16_kernel(const __bf16* __restrict__ src, uint4* __restrict__ dst, int n_tiles, int K, int mode,
                                 int hd, int tile_mul, int tile_off) {
    int KT = K / 32;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;  // (src_tile, kt, lane)
    long total = (long)n_tiles * KT * 64;
    if (idx >= total) return;
    int lane = idx & 63;
    long r = idx >> 6;
    int kt = r % KT;
    int st = r / KT;
    int dt = dst_tile_of(st, mode, hd, tile_mul, tile_off);
    const uint4* sp = (const uint4*)(src + ((size_t)(st * 16 + (lane & 15)) * K + kt * 32 + (lane >> 4) * 8));
    dst[((size_t)dt * KT + kt) * 64 + lane] = *sp;
}

__global__ void pack_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, int n_rows, int K, int mode, int hd,
                                int tile_mul, int tile_off) {
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)n_rows * K) return;
    int row = idx / K, k = idx % K;
    int dt = dst_tile_of(row / 16, mode, hd, tile_mul, tile_off);
    dst[((size_t)dt * 16 + (row & 15)) * K + k] = src[idx];
}

hipError_t launch_pack(int dtype, const void* src, void* dst, int n_rows, int K, int mode, int hd, int tile_mul,
                       int tile_off, hipStream_t s) {
    if (dtype == EE_BF16) {
        long total = (long)(n_rows / 16) * (K / 32) * 64;
        EE_LAUNCH(pack_bf16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), s, (const __bf16*)src,
                           (uint4*)dst, n_rows / 16, K, mode, hd, tile_mul, tile_off);
    } else {
        long total = (long)n_rows * K;
        EE_LAUNCH(pack_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), s, (const float*)src,
                           (float*)dst, n_rows, K, mode, hd, tile_mul, tile_off);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// embedding gather: x = E[token]; xg = st(x * g_next); ssq[slot][0] = sum x^2, ssq[slot][1..] = 0
// one workgroup per row
// ------------------------------------------------------------------------------------------------
template <typename ST>
__global__ void embed_kernel(const ST* __restrict__ embed, const int32_t* __restrict__ tokens, const SegDesc* __restrict__ desc,
                             int d, const float* __restrict__ g_next, float* __restrict__ x, ST* __restrict__ xg,
                             size_t xg_lo, float* __restrict__ ssq, int ssq_stride) {
    __shared__ float red[256];
    int r = blockIdx.x;
    int slot = desc->xrow[r];
    int tok = tokens[r];
    float s = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        float v = (float)embed[(size_t)tok * d + i];
        x[(size_t)slot * d + i] = v;
        store_split<ST>(xg + (size_t)slot * d + i, xg_lo, v * g_next[i]);
        s += v * v;
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    for (int i = threadIdx.x; i < ssq_stride; i += blockDim.x) ssq[(size_t)slot * ssq_stride + i] = (i == 0) ? red[0] : 0.f;
}

hipError_t launch_embed(int dtype, const void* embed, const int32_t* dev_tokens, const SegDesc* desc, int T, int d,
                        const float* g_next, float* x, void* xg, size_t xg_lo, float* ssq, int ssq_stride, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    if (dtype == EE_BF16)
        EE_LAUNCH(embed_kernel<__bf16>, dim3(T), dim3(256), s, (const __bf16*)embed, dev_tokens, desc, d, g_next, x,
                           (__bf16*)xg, xg_lo, ssq, ssq_stride);
    else
        EE_LAUNCH(embed_kernel<float>, dim3(T), dim3(256), s, (const float*)embed, dev_tokens, desc, d, g_next, x,
                           (float*)xg, xg_lo, ssq, ssq_stride);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// skinny GEMM: out[m][n] = r[m] * sum_k A[m][k] * W[n][k],  m < T <= MT*16
// A workgroup owns G consecutive 16-column tiles; its G*KS waves split K in KS parts.
// The result lands in LDS as out[MT*16][G*16] fp32 and is handed to the epilogue.
// ------------------------------------------------------------------------------------------------
struct GemmArgs {
    const void* W;
    int KT;  // K / 32 (bf16) ; K (fp32 path uses K directly)
    int K;
    const void* A;
    size_t a_lo;  // element offset of the lo term of A (bf16 only)
    int lda;
    const int32_t* arow;
    const float* ssq;
    int ssq_stride, ssq_n;
    float inv_d, eps;
    int T;
};

template <int G, int KS, int MT>
struct GemmSmem {
    float red[KS][G][MT][256];
    float out[MT * 16][G * 16];
    float rs[MT * 16];
};

template <int MT>
__device__ __forceinline__ void rms_scales(const GemmArgs& a, float* rs) {
    // r[m] = 1/sqrt(mean(x^2)+eps).  The sum of squares arrives as ssq_n partial sums (one per producing
    // workgroup); one wave per row adds them: lane-strided in order, then a fixed butterfly.
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    for (int m = wave; m < MT * 16; m += nw) {
        float r = 1.f;
        if (a.ssq != nullptr && m < a.T) {
            int slot = a.arow ? a.arow[m] : m;
            const float* p = a.ssq + (size_t)slot * a.ssq_stride;
            float s = 0.f;
            for (int i = lane; i < a.ssq_n; i += 64) s += p[i];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
            r = 1.0f / sqrtf(s * a.inv_d + a.eps);
        }
        if (lane == 0) rs[m] = r;
    }
}

template <int G, int KS, int MT>
__device__ __forceinline__ void gemm_mainloop_bf16(const GemmArgs& a, int tile0, GemmSmem<G, KS, MT>& sm) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g = wave / KS, ks = wave % KS;
    const int li = lane & 15, lg = lane >> 4;
    const int KT = a.KT;
    const int kt0 = (int)(((long)ks * KT) / KS), kt1 = (int)(((long)(ks + 1) * KT) / KS);
    const u32x4* wp = (const u32x4*)a.W + ((size_t)(tile0 + g) * KT + kt0) * 64 + lane;
    // Rows beyond T read row 0 again (always a valid address): their products are never looked at,
    // and an unpredicated load keeps the loop free of branches.
    const __bf16* ap[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int row = mt * 16 + li;
        if (row >= a.T) row = 0;
        int idx = a.arow ? a.arow[row] : row;
        ap[mt] = (const __bf16*)a.A + (size_t)idx * a.lda + (size_t)kt0 * 32 + lg * 8;
    }
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    // Rolling pipeline of D tiles (1 KB of weights each) per wave: a slot is refilled with the tile D
    // ahead as soon as its MFMAs are issued, so the wave always has about D KB of loads in flight.
    constexpr int D = MT == 1 ? 8 : (MT == 2 ? 6 : 4);
    u32x4 w[D], ah[MT][D], al[MT][D];
    const int n = kt1 - kt0;
    auto fill = [&](int u, int t) {  // slot u <- tile t (relative to kt0)
        w[u] = __builtin_nontemporal_load(wp + (size_t)t * 64);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            ah[mt][u] = *(const u32x4*)(ap[mt] + (size_t)t * 32);
            al[mt][u] = *(const u32x4*)(ap[mt] + a.a_lo + (size_t)t * 32);
        }
    };
    auto use = [&](int u) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, al[mt][u]),
                                                              __builtin_bit_cast(bf16x8, w[u]), acc[mt], 0, 0, 0);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ah[mt][u]),
                                                              __builtin_bit_cast(bf16x8, w[u]), acc[mt], 0, 0, 0);
        }
    };
    const int full = n / D, rem = n - full * D;
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < n) fill(u, u);
    for (int gI = 0; gI + 1 < full; ++gI) {  // steady state: every refill is in range
#pragma unroll
        for (int u = 0; u < D; ++u) {
            use(u);
            fill(u, (gI + 1) * D + u);
            __builtin_amdgcn_sched_barrier(0);  // keep the slot order: the wait before use(u+1) then covers one slot only
        }
    }
    if (full > 0) {  // last full group: refill only the slots the remainder needs
#pragma unroll
        for (int u = 0; u < D; ++u) {
            use(u);
            if (u < rem) fill(u, full * D + u);
        }
    }
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < rem) use(u);
    // accumulator layout: lane (lg, li) holds D[row = lg*4 + r][col = li]
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) sm.red[ks][g][mt][(lg * 4 + r) * 16 + li] = acc[mt][r];
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * MT * 256; idx += blockDim.x) {
        int e = idx & 255, mt = (idx >> 8) % MT, gg = idx / (256 * MT);
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < KS; ++k) s += sm.red[k][gg][mt][e];
        int m = mt * 16 + (e >> 4);
        sm.out[m][gg * 16 + (e & 15)] = s * sm.rs[m];
    }
    __syncthreads();
}

// fp32 path (tiny model, parity only): plain FMA loop, weights row-major [tile][16][K]
template <int G, int KS, int MT>
__device__ __forceinline__ void gemm_mainloop_f32(const GemmArgs& a, int tile0, GemmSmem<G, KS, MT>& sm) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < MT * 16 * G * 16; idx += blockDim.x) {
        int m = idx / (G * 16), c = idx % (G * 16);
        float s = 0.f;
        if (m < a.T) {
            int slot = a.arow ? a.arow[m] : m;
            const float* ar = (const float*)a.A + (size_t)slot * a.lda;
            const float* wr = (const float*)a.W + ((size_t)tile0 * 16 + c) * a.K;
            for (int k = 0; k < a.K; ++k) s = fmaf(ar[k], wr[k], s);
        }
        sm.out[m][c] = s * sm.rs[m];
    }
    __syncthreads();
}

template <typename ST, int G, int KS, int MT>
__device__ __forceinline__ void gemm_mainloop(const GemmArgs& a, int tile0, GemmSmem<G, KS, MT>& sm) {
#ifdef EE_EXP_NOSSQ
    for (int m = threadIdx.x; m < MT * 16; m += blockDim.x) sm.rs[m] = 1.f;
#else
    rms_scales<MT>(a, sm.rs);
#endif
    if constexpr (sizeof(ST) == 2)
        gemm_mainloop_bf16<G, KS, MT>(a, tile0, sm);  // (its first __syncthreads orders rs before use)
    else
        gemm_mainloop_f32<G, KS, MT>(a, tile0, sm);
}

// ---- epilogue 1: rotary embedding, q to the workspace, k and v into the paged cache
template <typename ST>
struct QkvArgs {
    ST* q;
    size_t q_lo;
    int d;
    const float2* rope_cs;
    ST* kv_layer;  // pool + layer * layer_stride
    size_t blk_stride;
    int H, hd, BT;
    const SegDesc* desc;
};

template <typename ST, int KS, int MT>
__global__ __launch_bounds__(2 * KS * 64) void gemm_qkv_kernel(GemmArgs a, QkvArgs<ST> e) {
    __shared__ GemmSmem<2, KS, MT> sm;
    gemm_mainloop<ST, 2, KS, MT>(a, blockIdx.x * 2, sm);
#ifdef EE_EXP_NOEPI
    if (sm.out[0][0] != 12345.f) return;
#endif
    const int per_part = e.H * (e.hd / 32);
    const int part = blockIdx.x / per_part;  // 0 q, 1 k, 2 v
    const int rem = blockIdx.x % per_part;
    const int h = rem / (e.hd / 32), c = rem % (e.hd / 32);
    const int half = e.hd / 2;
    for (int idx = threadIdx.x; idx < MT * 256; idx += blockDim.x) {
        int m = idx >> 4, i = idx & 15;
        if (m >= a.T) continue;
        float lo = sm.out[m][i], hi = sm.out[m][16 + i];
        int pos = e.desc->pos[m];
        if (part < 2) {
            float2 cs = e.rope_cs[(size_t)pos * half + c * 16 + i];
            float nlo = lo * cs.x - hi * cs.y;
            float nhi = hi * cs.x + lo * cs.y;
            lo = nlo;
            hi = nhi;
        }
        if (part == 0) {
            ST* qp = e.q + (size_t)m * e.d + h * e.hd + c * 16 + i;
            store_split<ST>(qp, e.q_lo, lo);
            store_split<ST>(qp + half, e.q_lo, hi);
        } else {
            ST* kp = e.kv_layer + (size_t)e.desc->kvblk[m] * e.blk_stride + (part == 2 ? (size_t)e.H * e.BT * e.hd : 0) +
                     ((size_t)h * e.BT + (pos % e.BT)) * e.hd + c * 16 + i;
            kp[0] = cvt_st<ST>(lo);
            kp[half] = cvt_st<ST>(hi);
        }
    }
}

// ---- epilogue 2: residual add; normalised-input operand(s) for what follows; sum-of-squares partial
template <typename ST>
struct ResidArgs {
    float* x;
    ST* xg;
    ST* xgh;
    size_t xs_lo;  // lo offset of xg and xgh
    float* ssq_out;
    int ssq_stride;
    const float* g_next;
    const float* g_head;
    int d;
    const SegDesc* desc;
};

template <typename ST, int KS, int MT>
__global__ __launch_bounds__(KS * 64) void gemm_resid_kernel(GemmArgs a, ResidArgs<ST> e) {
    __shared__ GemmSmem<1, KS, MT> sm;
    gemm_mainloop<ST, 1, KS, MT>(a, blockIdx.x, sm);
    const int n0 = blockIdx.x * 16;
#ifdef EE_EXP_NOEPI
    if (sm.out[0][0] != 12345.f) return;
#endif
    for (int idx = threadIdx.x; idx < MT * 256; idx += blockDim.x) {
        int m = idx >> 4, i = idx & 15;
        if (m >= a.T) continue;
        size_t o = (size_t)e.desc->xrow[m] * e.d + n0 + i;
        float v = e.x[o] + sm.out[m][i];
        e.x[o] = v;
        sm.out[m][i] = v;
        store_split<ST>(e.xg + o, e.xs_lo, v * e.g_next[n0 + i]);
        if (e.xgh) store_split<ST>(e.xgh + o, e.xs_lo, v * e.g_head[n0 + i]);
    }
    __syncthreads();
    for (int m = threadIdx.x; m < MT * 16; m += blockDim.x) {
        if (m >= a.T) continue;
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) s += sm.out[m][i] * sm.out[m][i];
        e.ssq_out[(size_t)e.desc->xrow[m] * e.ssq_stride + blockIdx.x] = s;
    }
}

// ---- epilogue 3: SwiGLU.  tile 2j holds gate features 16j.., tile 2j+1 the matching up features
template <typename ST, int KS, int MT>
__global__ __launch_bounds__(2 * KS * 64) void gemm_swiglu_kernel(GemmArgs a, ST* act, size_t act_lo, int F) {
    __shared__ GemmSmem<2, KS, MT> sm;
    gemm_mainloop<ST, 2, KS, MT>(a, blockIdx.x * 2, sm);
    for (int idx = threadIdx.x; idx < MT * 256; idx += blockDim.x) {
        int m = idx >> 4, i = idx & 15;
        if (m >= a.T) continue;
        float gt = sm.out[m][i], up = sm.out[m][16 + i];
        float sl = gt / (1.0f + expf(-gt));
        store_split<ST>(act + (size_t)m * F + blockIdx.x * 16 + i, act_lo, sl * up);
    }
}

// ---- epilogue 4: exit / final head.  Per workgroup: (max, arg max, sum exp) of its 32 logits per row.
// A one-workgroup kernel launched right after merges the partials in a fixed order and takes the exit
// decision (an in-kernel "last workgroup merges" scheme needs a device-wide fence in every workgroup,
// which costs more than the extra launch).
struct HeadArgs {
    HeadPartial* partials;  // [n_wg][EE_MAX_SEQS]
    float* logits;          // optional [row][V]
    int V;
};

__device__ __forceinline__ void merge_partial(float& m, float& s, int& i, float m2, float s2, int i2) {
    if (m2 > m || (m2 == m && i2 < i)) {
        s = s * expf(m - m2) + s2;
        m = m2;
        i = i2;
    } else {
        s = s + s2 * expf(m2 - m);
    }
}

template <typename ST, int KS, int MT>
__global__ __launch_bounds__(2 * KS * 64) void gemm_head_kernel(GemmArgs a, HeadArgs e) {
    __shared__ GemmSmem<2, KS, MT> sm;
    gemm_mainloop<ST, 2, KS, MT>(a, blockIdx.x * 2, sm);
    const int n0 = blockIdx.x * 32;
    if (e.logits) {
        for (int idx = threadIdx.x; idx < MT * 16 * 32; idx += blockDim.x) {
            int m = idx >> 5, c = idx & 31;
            if (m < a.T) e.logits[(size_t)m * e.V + n0 + c] = sm.out[m][c];
        }
    }
    for (int m = threadIdx.x; m < MT * 16; m += blockDim.x) {
        if (m >= a.T) continue;
        float mx = sm.out[m][0];
        int ix = 0;
        for (int c = 1; c < 32; ++c)
            if (sm.out[m][c] > mx) {
                mx = sm.out[m][c];
                ix = c;
            }
        float s = 0.f;
        for (int c = 0; c < 32; ++c) s += expf(sm.out[m][c] - mx);
        HeadPartial p;
        p.max = mx;
        p.sum = s;
        p.idx = n0 + ix;
        p.pad = 0;
        e.partials[(size_t)blockIdx.x * EE_MAX_SEQS + m] = p;
    }
}

// confidence = 1 / sum_i exp(z_i - z_max); exit iff confidence >= threshold (or always, for the final head)
__global__ __launch_bounds__(512) void head_merge_kernel(const HeadPartial* __restrict__ partials, int n_wg, int T, int mode,
                                                         float threshold, HeadResult* results,
                                                         const SegDesc* __restrict__ desc) {
    __shared__ float redm[512], reds[512];
    __shared__ int redi[512];
    // thread t folds workgroups t, t+512, ... in ascending order, then a fixed tree over the threads
    for (int m = 0; m < T; ++m) {
        float mx = -INFINITY, s = 0.f;
        int ix = 0x7fffffff;
        for (int w = threadIdx.x; w < n_wg; w += 512) {
            HeadPartial p = partials[(size_t)w * EE_MAX_SEQS + m];
            merge_partial(mx, s, ix, p.max, p.sum, p.idx);
        }
        redm[threadIdx.x] = mx;
        reds[threadIdx.x] = s;
        redi[threadIdx.x] = ix;
        __syncthreads();
        for (int o = 256; o > 0; o >>= 1) {
            if ((int)threadIdx.x < o) {
                float m1 = redm[threadIdx.x], s1 = reds[threadIdx.x];
                int i1 = redi[threadIdx.x];
                float m2 = redm[threadIdx.x + o], s2 = reds[threadIdx.x + o];
                int i2 = redi[threadIdx.x + o];
                if (s2 > 0.f || m2 > -INFINITY) merge_partial(m1, s1, i1, m2, s2, i2);
                redm[threadIdx.x] = m1;
                reds[threadIdx.x] = s1;
                redi[threadIdx.x] = i1;
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            float conf = 1.0f / reds[0];
            HeadResult r;
            r.token = redi[0];
            r.conf = conf;
            r.fired = (mode == HEAD_EMIT) || (conf >= threshold);
            r.pad = 0;
            results[desc->head_slot[m]] = r;
        }
        __syncthreads();
    }
}

// ---- host-side dispatch
static GemmArgs make_args(const GemmCommon& c) {
    GemmArgs a;
    a.W = c.W;
    a.K = c.K;
    a.KT = c.K / 32;
    a.A = c.A;
    a.a_lo = c.a_lo;
    a.lda = c.lda;
    a.arow = c.arow;
    a.ssq = c.ssq;
    a.ssq_stride = c.ssq_stride;
    a.ssq_n = c.ssq_n;
    a.inv_d = c.inv_d;
    a.eps = c.eps;
    a.T = c.T;
    return a;
}

static int mt_of(int T) { return T <= 16 ? 1 : (T <= 32 ? 2 : 4); }

#define EE_DISPATCH_MT(T, CALL)              \
    switch (mt_of(T)) {                      \
        case 1: { constexpr int MT = 1; CALL; } break; \
        case 2: { constexpr int MT = 2; CALL; } break; \
        default: { constexpr int MT = 4; CALL; } break; \
    }

constexpr int KS_QKV = 4, KS_RES = 8, KS_SWI = 4, KS_HEAD = 4;

int gemm_resid_tiles_per_wg() { return 1; }

hipError_t launch_gemm_qkv(const GemmCommon& c, void* q, size_t q_lo, const float* rope_cs, const KvGeom& kv, int layer,
                           hipStream_t s) {
    if (c.T <= 0) return hipSuccess;
    if (c.T > 64) return hipErrorInvalidValue;
    GemmArgs a = make_args(c);
    dim3 grid(c.N / 32), block(2 * KS_QKV * 64);
    if (c.dtype == EE_BF16) {
        QkvArgs<__bf16> e{(__bf16*)q, q_lo, c.N / 3, (const float2*)rope_cs, (__bf16*)kv.pool + (size_t)layer * kv.layer_stride,
                          kv.blk_stride, kv.H, kv.hd, kv.BT, c.desc};
        EE_DISPATCH_MT(c.T, EE_LAUNCH((gemm_qkv_kernel<__bf16, KS_QKV, MT>), grid, block, s, a, e));
    } else {
        QkvArgs<float> e{(float*)q, q_lo, c.N / 3, (const float2*)rope_cs, (float*)kv.pool + (size_t)layer * kv.layer_stride,
                         kv.blk_stride, kv.H, kv.hd, kv.BT, c.desc};
        EE_DISPATCH_MT(c.T, EE_LAUNCH((gemm_qkv_kernel<float, KS_QKV, MT>), grid, block, s, a, e));
    }
    return hipGetLastError();
}

hipError_t launch_gemm_resid(const GemmCommon& c, float* x, void* xg, void* xgh, size_t xs_lo, float* ssq_out,
                             const float* g_next, const float* g_head, int d, hipStream_t s) {
    if (c.T <= 0) return hipSuccess;
    if (c.T > 64) return hipErrorInvalidValue;
    GemmArgs a = make_args(c);
    dim3 grid(c.N / 16), block(KS_RES * 64);
    if (c.dtype == EE_BF16) {
        ResidArgs<__bf16> e{x, (__bf16*)xg, (__bf16*)xgh, xs_lo, ssq_out, c.ssq_stride, g_next, g_head, d, c.desc};
        EE_DISPATCH_MT(c.T, EE_LAUNCH((gemm_resid_kernel<__bf16, KS_RES, MT>), grid, block, s, a, e));
    } else {
        ResidArgs<float> e{x, (float*)xg, (float*)xgh, xs_lo, ssq_out, c.ssq_stride, g_next, g_head, d, c.desc};
        EE_DISPATCH_MT(c.T, EE_LAUNCH((gemm_resid_kernel<float, KS_RES, MT>), grid, block, s, a, e));
    }
    return hipGetLastError();
}

hipError_t launch_gemm_swiglu(const GemmCommon& c, void* act, size_t act_lo, int F, hipStream_t s) {
    if (c.T <= 0) return hipSuccess;
    if (c.T > 64) return hipErrorInvalidValue;
    GemmArgs a = make_args(c);
    dim3 grid(c.N / 32), block(2 * KS_SWI * 64);
    if (c.dtype == EE_BF16) {
        EE_DISPATCH_MT(c.T, EE_LAUNCH((gemm_swiglu_kernel<__bf16, KS_SWI, MT>), grid, block, s, a, (__bf16*)act, act_lo, F));
    } else {
        EE_DISPATCH_MT(c.T, EE_LAUNCH((gemm_swiglu_kernel<float, KS_SWI, MT>), grid, block, s, a, (float*)act, act_lo, F));
    }
    return hipGetLastError();
}

hipError_t launch_gemm_head(const GemmCommon& c, HeadPartial* partials, int32_t* counter, float* logits, int mode,
                            float threshold, HeadResult* results, hipStream_t s) {
    if (c.T <= 0) return hipSuccess;
    if (c.T > 64) return hipErrorInvalidValue;
    GemmArgs a = make_args(c);
    (void)counter;
    HeadArgs e{partials, logits, c.N};
    dim3 grid(c.N / 32), block(2 * KS_HEAD * 64);
    if (c.dtype == EE_BF16) {
        EE_DISPATCH_MT(c.T, EE_LAUNCH((gemm_head_kernel<__bf16, KS_HEAD, MT>), grid, block, s, a, e));
    } else {
        EE_DISPATCH_MT(c.T, EE_LAUNCH((gemm_head_kernel<float, KS_HEAD, MT>), grid, block, s, a, e));
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    EE_LAUNCH(head_merge_kernel, dim3(1), dim3(512), s, partials, (int)grid.x, c.T, mode, threshold, results, c.desc);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// attention, reference-grade kernel: one workgroup per (row, head); the row at position p attends to
// cache positions 0..p of its sequence (which includes the rows before it in this launch: their K,V
// were written by the QKV kernel).  Online soft-max over chunks of 1024 positions.
// ------------------------------------------------------------------------------------------------
template <typename ST>
__device__ __forceinline__ const ST* kv_ptr(const ST* layer_base, const KvGeom& kv, const int32_t* bt, int which, int h,
                                             int pos) {
    int blk = bt[pos / kv.BT];
    return layer_base + (size_t)blk * kv.blk_stride + (which ? (size_t)kv.H * kv.BT * kv.hd : 0) +
           ((size_t)h * kv.BT + (pos % kv.BT)) * kv.hd;
}

__device__ __forceinline__ float block_reduce(float v, float* red, bool is_max) {
    red[threadIdx.x] = v;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) {
            float b = red[threadIdx.x + o];
            red[threadIdx.x] = is_max ? fmaxf(red[threadIdx.x], b) : red[threadIdx.x] + b;
        }
        __syncthreads();
    }
    float r = red[0];
    __syncthreads();
    return r;
}

template <typename ST>
__global__ __launch_bounds__(256) void attn_simple_kernel(const ST* __restrict__ q, ST* __restrict__ out,
                                                          size_t io_lo, const SegDesc* __restrict__ desc,
                                                          const int32_t* __restrict__ btab, KvGeom kv,
                                                          const ST* __restrict__ layer_base, int d) {
    __shared__ float qs[128];
    __shared__ float sc[1024];
    __shared__ float red[256];
    const int r = blockIdx.x, h = blockIdx.y, hd = kv.hd;
    const int pos = desc->pos[r];
    const int32_t* bt = btab + (size_t)desc->rseq[r] * kv.max_blocks_per_seq;
    const float scale = 1.0f / sqrtf((float)hd);
    for (int i = threadIdx.x; i < hd; i += 256) qs[i] = load_split<ST>(q + (size_t)r * d + h * hd + i, io_lo);
    __syncthreads();
    float m = -INFINITY, l = 0.f, acc = 0.f;
    const int n_ctx = pos + 1;
    for (int j0 = 0; j0 < n_ctx; j0 += 1024) {
        int nj = min(1024, n_ctx - j0);
        float cmax = -INFINITY;
        for (int jj = threadIdx.x; jj < nj; jj += 256) {
            const ST* kp = kv_ptr(layer_base, kv, bt, 0, h, j0 + jj);
            float s = 0.f;
            for (int c = 0; c < hd; ++c) s = fmaf(qs[c], (float)kp[c], s);
            s *= scale;
            sc[jj] = s;
            cmax = fmaxf(cmax, s);
        }
        cmax = block_reduce(cmax, red, true);
        float m_new = fmaxf(m, cmax);
        float psum = 0.f;
        for (int jj = threadIdx.x; jj < nj; jj += 256) {
            float p = expf(sc[jj] - m_new);
            sc[jj] = p;
            psum += p;
        }
        psum = block_reduce(psum, red, false);
        float corr = expf(m - m_new);  // exp(-inf) = 0 on the first chunk
        l = l * corr + psum;
        if ((int)threadIdx.x < hd) {
            float a2 = 0.f;
            for (int jj = 0; jj < nj; ++jj) a2 = fmaf(sc[jj], (float)kv_ptr(layer_base, kv, bt, 1, h, j0 + jj)[threadIdx.x], a2);
            acc = acc * corr + a2;
        }
        m = m_new;
        __syncthreads();
    }
    if ((int)threadIdx.x < hd) store_split<ST>(out + (size_t)r * d + h * hd + threadIdx.x, io_lo, acc / l);
}

// ------------------------------------------------------------------------------------------------
// attention, bf16 model: ragged multi-query decode attention over the paged cache with MFMA.
// One workgroup = (query tile of <= 16 consecutive rows of one sequence, head, KV split); its 4 waves
// take the split's 32-position tiles round-robin.  Per tile a wave computes S^T = K Q^T (K rows come
// straight from the cache as MFMA A operands: 64 contiguous bytes per lane), applies the causal mask
// (only the last rows of the context differ between the queries of a tile), keeps an online soft-max
// per query, stages the V tile through LDS (coalesced 16-byte loads in, transposed 2-byte reads out)
// and accumulates O^T += V^T P^T, where P^T is already in B-operand layout in the S^T registers.
// q and P are fed as two bf16 terms each (hi + lo), so only K and V carry bf16 rounding.
// Partials of the KV splits are merged by attn_merge_kernel in a fixed order.
// ------------------------------------------------------------------------------------------------
constexpr int ATT_MAX_SPLITS = 16;

__host__ __device__ inline int att_part_stride(int hd) { return 32 + 16 * hd; }

template <int HD>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const __bf16* __restrict__ q, size_t q_lo, __bf16* __restrict__ out,
                                                        size_t out_lo, const SegDesc* __restrict__ desc,
                                                        const int32_t* __restrict__ btab, KvGeom kv,
                                                        const __bf16* __restrict__ layer_base, int d, int NS,
                                                        float* __restrict__ part) {
    constexpr int KK = HD / 32, CG = HD / 16, VST = HD + 4;  // LDS row stride (elements): HD/2 + 2 dwords, conflict-free
    constexpr int STAGE_BYTES = 4 * 32 * VST * 2;
    constexpr int COMB_BYTES = (4 * 16 * (HD + 1) + 128) * 4;
    __shared__ __attribute__((aligned(16))) unsigned char smem[STAGE_BYTES > COMB_BYTES ? STAGE_BYTES : COMB_BYTES];
    const int qt = blockIdx.x / kv.H, h = blockIdx.x % kv.H, split = blockIdx.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, li = lane & 15, lg = lane >> 4;
    const int row0 = desc->qt_row0[qt], nq = desc->qt_nq[qt];
    const int pos0 = desc->pos[row0];
    const int ctx = pos0 + nq;
    const int32_t* bt = btab + (size_t)desc->rseq[row0] * kv.max_blocks_per_seq;
    const int n_tiles = (ctx + 31) >> 5;
    const int tps = (n_tiles + NS - 1) / NS;
    const int t_lo = split * tps, t_hi = min(n_tiles, t_lo + tps);
    const bool qvalid = li < nq;

    bf16x8 qh[KK], ql[KK];
    {
        const __bf16* qp = q + (size_t)(row0 + (qvalid ? li : 0)) * d + h * HD + lg * (HD / 4);
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            u32x4 a = qvalid ? *(const u32x4*)(qp + kk * 8) : zero;
            u32x4 b = qvalid ? *(const u32x4*)(qp + q_lo + kk * 8) : zero;
            qh[kk] = __builtin_bit_cast(bf16x8, a);
            ql[kk] = __builtin_bit_cast(bf16x8, b);
        }
    }
    const float scale = 1.0f / sqrtf((float)HD);
    float m_run = -INFINITY, l_run = 0.f;
    f32x4 o[CG];
#pragma unroll
    for (int c = 0; c < CG; ++c) o[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    __bf16* vs = (__bf16*)smem + (size_t)wave * 32 * VST;

    for (int t = t_lo + wave; t < t_hi; t += 4) {
        const int tb = t << 5;
        const int blk = bt[tb / kv.BT];
        const __bf16* kbase = layer_base + (size_t)blk * kv.blk_stride + ((size_t)h * kv.BT + (tb % kv.BT)) * HD;
        const __bf16* vbase = kbase + (size_t)kv.H * kv.BT * HD;
        // scores, transposed: rows = positions, columns = queries
        f32x4 sacc[2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            sacc[sub] = f32x4{0.f, 0.f, 0.f, 0.f};
            const __bf16* kp = kbase + (size_t)(sub * 16 + li) * HD + lg * (HD / 4);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                bf16x8 kf = __builtin_bit_cast(bf16x8, *(const u32x4*)(kp + kk * 8));
                sacc[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, ql[kk], sacc[sub], 0, 0, 0);
                sacc[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qh[kk], sacc[sub], 0, 0, 0);
            }
        }
        // V tile -> LDS (rows beyond the context are zeroed: their probabilities are zero, their bits unknown)
#pragma unroll
        for (int ci = lane; ci < 32 * HD / 8; ci += 64) {
            int p = ci / (HD / 8), c8 = ci % (HD / 8);
            u32x4 v = {0u, 0u, 0u, 0u};
            if (tb + p < ctx) v = *(const u32x4*)(vbase + (size_t)p * HD + c8 * 8);
            uint2* dst = (uint2*)(vs + p * VST + c8 * 8);
            dst[0] = make_uint2(v.x, v.y);
            dst[1] = make_uint2(v.z, v.w);
        }
        // causal mask + online soft-max per query (column li); this lane holds positions lg*4+r of each half
        float pv[8];
        float tmax = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int pa = tb + (e >> 2) * 16 + lg * 4 + (e & 3);
            float val = (qvalid && pa <= pos0 + li) ? sacc[e >> 2][e & 3] * scale : -INFINITY;
            pv[e] = val;
            tmax = fmaxf(tmax, val);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax);
        float corr = 1.f, psum = 0.f;
        if (m_new == -INFINITY) {
#pragma unroll
            for (int e = 0; e < 8; ++e) pv[e] = 0.f;
        } else {
            corr = expf(m_run - m_new);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pv[e] = expf(pv[e] - m_new);
                psum += pv[e];
            }
        }
        psum += __shfl_xor(psum, 16);
        psum += __shfl_xor(psum, 32);
        l_run = l_run * corr + psum;
        m_run = m_new;
        bf16x8 ph, pl;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            __bf16 hi = (__bf16)pv[e];
            ph[e] = hi;
            pl[e] = (__bf16)(pv[e] - (float)hi);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int c = 0; c < CG; ++c) {
            bf16x8 vf;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int pe = (e >> 2) * 16 + lg * 4 + (e & 3);
                vf[e] = vs[pe * VST + c * 16 + li];
            }
            o[c] = o[c] * corr;
            o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pl, o[c], 0, 0, 0);
            o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, ph, o[c], 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // combine the 4 waves (fixed order)
    __syncthreads();
    float* wO = (float*)smem;  // [4][16][HD+1]
    float* wm = wO + 4 * 16 * (HD + 1);
    float* wl = wm + 64;
#pragma unroll
    for (int c = 0; c < CG; ++c)
#pragma unroll
        for (int r = 0; r < 4; ++r) wO[(wave * 16 + li) * (HD + 1) + c * 16 + lg * 4 + r] = o[c][r];
    if (lg == 0) {
        wm[wave * 16 + li] = m_run;
        wl[wave * 16 + li] = l_run;
    }
    __syncthreads();
    float* pbase = part + ((size_t)(qt * kv.H + h) * NS + split) * att_part_stride(HD);
    for (int idx = threadIdx.x; idx < 16 * HD; idx += 256) {
        int qq = idx / HD, cc = idx % HD;
        if (qq >= nq) continue;
        float M = fmaxf(fmaxf(wm[qq], wm[16 + qq]), fmaxf(wm[32 + qq], wm[48 + qq]));
        float O = 0.f, L = 0.f;
        if (M > -INFINITY) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                float f = expf(wm[w * 16 + qq] - M);
                O += f * wO[(w * 16 + qq) * (HD + 1) + cc];
                L += f * wl[w * 16 + qq];
            }
        }
        if (NS == 1) {
            store_split<__bf16>(out + (size_t)(row0 + qq) * d + h * HD + cc, out_lo, O / L);
        } else {
            pbase[32 + qq * HD + cc] = O;
            if (cc == 0) {
                pbase[qq] = M;
                pbase[16 + qq] = L;
            }
        }
    }
}

template <int HD>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ part, int NS, __bf16* __restrict__ out,
                                                         size_t out_lo, const SegDesc* __restrict__ desc, int H, int d) {
    const int qt = blockIdx.x / H, h = blockIdx.x % H;
    const int row0 = desc->qt_row0[qt], nq = desc->qt_nq[qt];
    const float* pb = part + (size_t)(qt * H + h) * NS * att_part_stride(HD);
    for (int idx = threadIdx.x; idx < nq * HD; idx += 256) {
        int qq = idx / HD, cc = idx % HD;
        float M = -INFINITY;
        for (int s = 0; s < NS; ++s) M = fmaxf(M, pb[(size_t)s * att_part_stride(HD) + qq]);
        float O = 0.f, L = 0.f;
        for (int s = 0; s < NS; ++s) {
            const float* ps = pb + (size_t)s * att_part_stride(HD);
            float ms = ps[qq];
            if (ms == -INFINITY) continue;
            float f = expf(ms - M);
            O += f * ps[32 + qq * HD + cc];
            L += f * ps[16 + qq];
        }
        store_split<__bf16>(out + (size_t)(row0 + qq) * d + h * HD + cc, out_lo, O / L);
    }
}

size_t attention_part_floats(int max_rows, int H, int hd) {
    size_t entries = (size_t)max_rows * H;
    if (entries < 1024) entries = 1024;
    return entries * att_part_stride(hd);
}

template <int HD>
static hipError_t launch_attention_mfma(const void* q, void* out, size_t io_lo, const SegDesc* desc, int n_qt, const int32_t* btab,
                                        const KvGeom& kv, int layer, int d, float* part, int max_ctx, hipStream_t s) {
    int wgs = n_qt * kv.H;
    int NS = 1024 / wgs;
    int by_len = ((max_ctx + 31) / 32 + 3) / 4;  // at least ~4 tiles (one per wave) per split
    if (NS > by_len) NS = by_len;
    if (NS > ATT_MAX_SPLITS) NS = ATT_MAX_SPLITS;
    if (NS < 1) NS = 1;
    const __bf16* lb = (const __bf16*)kv.pool + (size_t)layer * kv.layer_stride;
    EE_LAUNCH(attn_mfma_kernel<HD>, dim3(wgs, NS), dim3(256), s, (const __bf16*)q, io_lo, (__bf16*)out, io_lo, desc,
                       btab, kv, lb, d, NS, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || NS == 1) return e;
    EE_LAUNCH(attn_merge_kernel<HD>, dim3(wgs), dim3(256), s, (const float*)part, NS, (__bf16*)out, io_lo, desc, kv.H, d);
    return hipGetLastError();
}

hipError_t launch_attention(int dtype, const void* q, void* out, size_t io_lo, const SegDesc* desc, int T, int n_qt, const int32_t* btab,
                            const KvGeom& kv, int layer, int d, float* part, int32_t* counters, int max_ctx,
                            hipStream_t s) {
    (void)counters;
    if (T <= 0) return hipSuccess;
    if (dtype == EE_BF16) {
        switch (kv.hd) {
            case 32: return launch_attention_mfma<32>(q, out, io_lo, desc, n_qt, btab, kv, layer, d, part, max_ctx, s);
            case 64: return launch_attention_mfma<64>(q, out, io_lo, desc, n_qt, btab, kv, layer, d, part, max_ctx, s);
            case 128: return launch_attention_mfma<128>(q, out, io_lo, desc, n_qt, btab, kv, layer, d, part, max_ctx, s);
            default: return hipErrorInvalidValue;
        }
    }
    dim3 grid(T, kv.H), block(256);
    EE_LAUNCH(attn_simple_kernel<float>, grid, block, s, (const float*)q, (float*)out, io_lo, desc, btab, kv,
                       (const float*)kv.pool + (size_t)layer * kv.layer_stride, d);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// cache export (tests): K,V of positions [pos0, pos0+n) of one layer as fp32 [n][d]
// ------------------------------------------------------------------------------------------------
template <typename ST>
__global__ void kv_gather_kernel(KvGeom kv, const ST* __restrict__ layer_base, const int32_t* __restrict__ bt, int pos0, int n,
                                 float* __restrict__ k_out, float* __restrict__ v_out) {
    int d = kv.H * kv.hd;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)n * d) return;
    int t = idx / d, c = idx % d;
    int h = c / kv.hd, i = c % kv.hd;
    k_out[idx] = (float)kv_ptr(layer_base, kv, bt, 0, h, pos0 + t)[i];
    v_out[idx] = (float)kv_ptr(layer_base, kv, bt, 1, h, pos0 + t)[i];
}

hipError_t launch_kv_gather(int dtype, const KvGeom& kv, int layer, const int32_t* btab_seq, int pos0, int n,
                            float* k_out, float* v_out, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    long total = (long)n * kv.H * kv.hd;
    dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (dtype == EE_BF16)
        EE_LAUNCH(kv_gather_kernel<__bf16>, grid, block, s, kv, (const __bf16*)kv.pool + (size_t)layer * kv.layer_stride,
                           btab_seq, pos0, n, k_out, v_out);
    else
        EE_LAUNCH(kv_gather_kernel<float>, grid, block, s, kv, (const float*)kv.pool + (size_t)layer * kv.layer_stride,
                           btab_seq, pos0, n, k_out, v_out);
    return hipGetLastError();
}

}  // namespace ee
